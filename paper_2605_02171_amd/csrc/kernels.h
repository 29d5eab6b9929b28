// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qv {

constexpr uint32_t EMPTY_ID = 0xFFFFFFFFu;
// encodings (values of QV_ENC_* in the C ABI): Sign-Magnitude, and the two of the paper's ablation
constexpr int ENC_SM = 0, ENC_SIGN1 = 1, ENC_SQ2 = 2;
inline int code_row_words(int nw, int encoding) { return (encoding == ENC_SIGN1 ? 1 : 2) * nw; }
__device__ inline int code_row_words_dev(int nw, int encoding) { return (encoding == ENC_SIGN1 ? 1 : 2) * nw; }
constexpr uint32_t QV_STATUS_NONFINITE_BIT = 1u;
constexpr uint32_t QV_STATUS_VISITED_FULL_BIT = 2u;
constexpr uint32_t QV_STATUS_BAD_EDGE_BIT = 4u;
constexpr uint32_t QV_STATUS_TIMEOUT_BIT = 8u;

// Split layout of Sign-Magnitude code rows longer than one 128-byte line (a rearrangement of the same words, same
// total size).  First array: per row the whole sign plane, then the first split_k1(nw) magnitude words, which fill the
// row up to a multiple of 128 bytes (split_stride1(nw) words).  Second array: the remaining magnitude words, dense.
// The sign plane alone bounds a distance from below, so the search reads the second array only for neighbours that
// the bound does not already keep out of the list.
constexpr int split_stride1(int nw) { return (nw + 15) / 16 * 16; }
constexpr int split_k1(int nw) { return split_stride1(nw) - nw < nw ? split_stride1(nw) - nw : nw; }
constexpr int split_stride2(int nw) { return nw - split_k1(nw); }
// widths the search kernel is compiled for in this layout, with the lanes per row it uses there (0: none)
constexpr int split_lanes_per_row(int nw) { return nw == 12 ? 2 : ((nw == 16 || nw == 24) ? 4 : 0); }

struct SearchParams {
    const uint32_t* adj;     // [n][R]
    const uint64_t* codes;   // [n] rows of code_row_words(nw, encoding) words, row_stride words apart
    const uint64_t* codes1;  // split layout (see above), or null: [n][split_stride1(nw)] ...
    const uint64_t* codes2;  // ... and [n][split_stride2(nw)]
    const uint64_t* qcodes;  // [nq][code_row_words(nw, encoding)]
    int encoding;            // ENC_*
    int row_stride;          // 64-bit words between the rows of `codes` (even, >= the row's words); qcodes are dense
    int64_t n;
    int64_t nq;
    int nw;                  // 64-bit words per bit-plane as stored (codes and qcodes alike; >= ceil(d / 64), zero padded)
    int R;
    uint32_t entry;
    int ef;
    uint32_t vis_slots;      // slots of the visited table (see plan_visited_table)
    int vis_bucket_bits;     // 32-bit entries: log2(number of 4-slot buckets)
    uint32_t vis_regions;    // > 0: 16-bit entries, table cut into this many parts ...
    uint32_t vis_region_buckets;  // ... of this many 8-tag buckets each (see plan_visited_table)
    int vis_cache;           // 0: the table never forgets an id (stops taking ids when nearly full); 1: ids displace each other
    const uint32_t* order;   // [nq] launch order: workgroup b runs query order[b]; null: query b
    const uint32_t* qstatus; // [nq] status words of the query encode, or null: a query flagged QV_STATUS_NONFINITE_BIT is
                             // not searched (its code is unspecified) and returns an empty list
    // outputs
    uint32_t* cand_ids;      // [nq][ef]
    uint32_t* cand_dist;     // [nq][ef]
    uint32_t* n_cand;        // [nq]
    uint32_t* n_expanded;    // [nq] or null
    uint32_t* n_evals;       // [nq] or null
    uint32_t* status;        // [nq] or null
    uint32_t* visit_order;   // [nq][visit_cap] or null
    int64_t visit_cap;
    // Stage 2 inside the search kernel (rr_vecs != null; beams of up to 128 entries): the wave that finished a query
    // scores its final list at once, so that this streaming work fills the time in which other waves wait for their
    // gathers.  cand_ids / cand_dist / n_cand may then be null.
    // Stage 2 by other waves of the same launch (rr_ticket != null, together with rr_vecs): the grid has 2 * nq
    // workgroups; each takes a ticket from *rr_ticket when it starts.  Tickets below nq search query order[ticket];
    // ticket nq + j scores the final list of query order[j] once rr_done says that it is in memory.  Whoever holds
    // a scoring ticket started after every search ticket had been taken by a workgroup that is already running, so
    // the wait always ends.  The scoring waves arrive when the last searches are under way and fill the memory system
    // the emptier end of the batch leaves idle.  The list (cand_ids, n_cand: required) and the flag travel between
    // the compute dies in device-coherent stores and loads; no cache is flushed or invalidated for them.
    uint32_t* rr_ticket;      // [1], 0 before the launch
    uint32_t* rr_done;        // [nq], 0 before the launch
    uint32_t rr_spin_limit;   // polls (of about two microseconds) a scoring wave waits for its list before it gives up
                              // and reports QV_STATUS_TIMEOUT_BIT with an empty result
    const float* rr_queries;  // [nq][rr_d]
    const float* rr_vecs;     // [n][rr_d]
    int rr_d, rr_k;
    uint32_t* rr_ids;         // [nq][rr_k]
    float* rr_scores;         // [nq][rr_k]
};

struct RerankParams {
    const float* queries;    // [nq][d]
    const float* vecs;       // [n][d]
    const uint32_t* cand_ids;  // [nq][ef]
    const uint32_t* n_cand;  // [nq]
    int64_t nq;
    int d;
    int ef;
    int k;
    uint32_t* ids;           // [nq][k]
    float* scores;           // [nq][k]
};

hipError_t launch_encode(const float* x, int64_t n, int d, int encoding, uint64_t* codes, uint32_t* status,
                         hipStream_t stream);
// dense code rows (planes of nw words) -> rows `stride` words apart whose planes are plane_words long (zero filled)
hipError_t launch_pad_codes(const uint64_t* codes, int64_t n, int nw, int planes, int plane_words, int stride, uint64_t* out,
                            hipStream_t stream);
hipError_t launch_bq_distance(const uint64_t* a, const int64_t* ia, const uint64_t* b, const int64_t* ib,
                              int64_t npairs, int d, int encoding, uint32_t* out, hipStream_t stream);
// dense Sign-Magnitude rows -> the two arrays of the split layout
hipError_t launch_split_codes(const uint64_t* codes, int64_t n, int nw, uint64_t* out1, uint64_t* out2, hipStream_t stream);
hipError_t launch_gather_probe(const uint64_t* codes, int d, const uint32_t* ids, int64_t n_ids, uint64_t* sink,
                               hipStream_t stream);
int64_t bq_scan_chunk_rows(int64_t n);
hipError_t launch_bq_scan(const uint64_t* codes, int64_t n, int d, int encoding, const uint64_t* qcodes, int64_t nq, int K,
                          uint64_t* partial, uint32_t* ids, uint32_t* dist, hipStream_t stream);
hipError_t launch_topk_overlap(const uint32_t* a, const uint32_t* b, int64_t nq, int K, uint32_t* out,
                               hipStream_t stream);
// smallest plane width >= nw the construction kernels are compiled for with this encoding; 0 if there is none
int build_width_at_least(int nw, int encoding);
size_t build_workspace_bytes(int64_t n, int nw, int encoding, int R, int L, int64_t max_batch);
hipError_t build_graph(const uint64_t* codes, int64_t n, int d, int encoding, int R, int L, double alpha, uint32_t entry,
                       int64_t max_batch, uint32_t* adj, void* workspace, hipStream_t stream);
// smallest plane width >= nw the search kernel is compiled for with this encoding; 0 if there is none
int search_compiled_width_at_least(int nw, int encoding);
// lanes_per_row: 0 = pick from the shape
hipError_t launch_beam_search(const SearchParams& p, int lanes_per_row, hipStream_t stream);
// Fills order[nq] with a launch order of the queries: those whose code is farthest from the entry node's code
// first (approximately).  Returns false (nothing launched) when the batch is too small or too large for it to
// matter; then the caller passes no order.
// rr_ticket / rr_done (may be null): cleared by the same kernel for a launch with Stage 2 in other waves
bool launch_query_order(const SearchParams& p, uint32_t* order, uint32_t* rr_ticket, uint32_t* rr_done, hipStream_t stream,
                        hipError_t* err);
// LDS bytes one query of the search kernel needs: visited table, two 64-entry lists, the merge scatter area
// (64 keys per pool register of a lane, plus 64), the query code
inline int beam_search_pool_registers(int ef) {
    const int p = (ef + 63) / 64;
    return p <= 1 ? 1 : (p <= 2 ? 2 : (p <= 4 ? 4 : (p <= 8 ? 8 : 16)));
}
inline size_t beam_search_lds_bytes(int nw, uint32_t vis_slots, bool narrow, int ef) {
    return (size_t)vis_slots * (narrow ? 2 : 4) + 64 * 4 * 2 + (size_t)(64 * beam_search_pool_registers(ef) + 64) * 8 +
           (size_t)nw * 24 + 16;
}
void plan_visited_table(SearchParams& p, uint32_t slots, bool allow_narrow, bool cache);
hipError_t launch_rerank(const RerankParams& p, hipStream_t stream);

}  // namespace qv
