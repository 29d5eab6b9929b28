// C ABI of the library (see include/quiver.h): argument checks, workspace carving, launches.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>

#include "../../include/quiver.h"
#include "kernels.h"

static_assert(QV_STATUS_NONFINITE == qv::QV_STATUS_NONFINITE_BIT, "status bits");
static_assert(QV_STATUS_VISITED_FULL == qv::QV_STATUS_VISITED_FULL_BIT, "status bits");
static_assert(QV_STATUS_BAD_EDGE == qv::QV_STATUS_BAD_EDGE_BIT, "status bits");
static_assert(QV_STATUS_TIMEOUT == qv::QV_STATUS_TIMEOUT_BIT, "status bits");
static_assert(QV_EMPTY == qv::EMPTY_ID, "empty id");

namespace {

thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e, const char* where) {
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", where, hipGetErrorString(e));
    return QV_ERR_HIP;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct WorkspaceLayout {
    size_t qcodes, qcodes_wide, cand_ids, cand_dist, n_cand, order, qstatus, rr_done, rr_ticket, total;
};

// widest plane (64-bit words) an index may store for vectors of nw words per plane: half as much again, plus two
inline int max_plane_words(int nw) { return nw + nw / 2 + 2; }

WorkspaceLayout layout(int64_t nq, int d, int ef) {
    WorkspaceLayout L;
    size_t off = 0;
    L.qcodes = off;    off = align_up(off + (size_t)nq * qv_code_words(d) * 8, 256);
    L.qcodes_wide = off; off = align_up(off + (size_t)nq * 2 * max_plane_words((d + 63) / 64) * 8, 256);   // queries in a widened index layout
    L.cand_ids = off;  off = align_up(off + (size_t)nq * ef * 4, 256);
    L.cand_dist = off; off = align_up(off + (size_t)nq * ef * 4, 256);
    L.n_cand = off;    off = align_up(off + (size_t)nq * 4, 256);
    L.order = off;     off = align_up(off + (size_t)nq * 4, 256);
    L.qstatus = off;   off = align_up(off + (size_t)nq * 4, 256);
    L.rr_done = off;   off = align_up(off + (size_t)nq * 4, 256);
    L.rr_ticket = off; off += 256;
    L.total = off;
    return L;
}

}  // namespace

struct qv_timer {
    int max_calls;
    int used;
    hipEvent_t* ev;  // 4 per call: start, after encode, after search, after rerank
};

struct qv_index {
    int64_t n;
    int d, R;
    const uint32_t* adj;
    const uint64_t* codes;
    const float* vecs;
    uint32_t entry;
    int visited_slots;  // <= 0: choose from ef
    int lanes_per_row;  // <= 0: choose from d
    int table_format;   // 0: 16-bit visited entries when the graph is small enough; 32: always 32-bit
    int visited_mode;   // 0: choose from ef; QV_VISITED_EXACT; QV_VISITED_CACHE
    int rerank_mode;    // 0: choose; QV_RERANK_SEPARATE; QV_RERANK_FUSED; QV_RERANK_TAIL
    bool vecs_on_device;  // false: the float32 vectors live in host memory the device can address
    int encoding;       // QV_ENC_*: what `codes` holds and what the queries are encoded to
    int code_plane_words;  // 64-bit words per bit-plane as stored in `codes`; 0: ceil(d / 64)
    int code_stride;    // 64-bit words between rows of `codes`; 0: dense
    const uint64_t* split1;  // the codes again in the split layout (qv_index_set_split_codes), or null
    const uint64_t* split2;
    qv_timer* timer;
};

extern "C" {

static bool enc_ok(int encoding) { return encoding == QV_ENC_SM || encoding == QV_ENC_SIGN1 || encoding == QV_ENC_SQ2; }

int qv_code_words(int d) { return qv_code_words_enc(d, QV_ENC_SM); }

int qv_code_words_enc(int d, int encoding) {
    return (d < 1 || d > QV_MAX_DIM || !enc_ok(encoding)) ? 0 : qv::code_row_words((d + 63) / 64, encoding);
}

int qv_encode(const float* x, int64_t n, int d, uint64_t* codes, uint32_t* status, void* stream) {
    return qv_encode_enc(x, n, d, QV_ENC_SM, codes, status, stream);
}

int qv_encode_enc(const float* x, int64_t n, int d, int encoding, uint64_t* codes, uint32_t* status, void* stream) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (n < 0 || n > (1ll << 32) || !enc_ok(encoding)) return QV_ERR_INVALID_ARG;
    if (n == 0) return QV_OK;
    if (!x || !codes) return QV_ERR_NULL;
    hipError_t e = qv::launch_encode(x, n, d, encoding, codes, status, (hipStream_t)stream);
    return e == hipSuccess ? QV_OK : hip_fail(e, "encode launch");
}

int qv_bq_distance(const uint64_t* codes_a, const int64_t* ia, const uint64_t* codes_b, const int64_t* ib,
                   int64_t npairs, int d, uint32_t* out, void* stream) {
    return qv_bq_distance_enc(codes_a, ia, codes_b, ib, npairs, d, QV_ENC_SM, out, stream);
}

int qv_bq_distance_enc(const uint64_t* codes_a, const int64_t* ia, const uint64_t* codes_b, const int64_t* ib,
                       int64_t npairs, int d, int encoding, uint32_t* out, void* stream) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (npairs < 0 || !enc_ok(encoding)) return QV_ERR_INVALID_ARG;
    if (npairs == 0) return QV_OK;
    if (!codes_a || !codes_b || !ia || !ib || !out) return QV_ERR_NULL;
    hipError_t e = qv::launch_bq_distance(codes_a, ia, codes_b, ib, npairs, d, encoding, out, (hipStream_t)stream);
    return e == hipSuccess ? QV_OK : hip_fail(e, "bq_distance launch");
}

int qv_gather_probe(const uint64_t* codes, int64_t n, int d, const uint32_t* ids, int64_t n_ids, uint64_t* sink,
                    void* stream) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (n < 1 || n_ids < 0) return QV_ERR_INVALID_ARG;
    if (!codes || !ids || !sink) return QV_ERR_NULL;
    hipError_t e = qv::launch_gather_probe(codes, d, ids, n_ids, sink, (hipStream_t)stream);
    return e == hipSuccess ? QV_OK : hip_fail(e, "gather probe launch");
}

size_t qv_bq_scan_workspace_bytes(int64_t n, int64_t nq, int K) {
    if (n < 0 || nq < 0 || K < 1 || K > QV_MAX_SCAN_K) return 0;
    const int64_t chunk = qv::bq_scan_chunk_rows(n);
    const int64_t nchunks = n > 0 ? (n + chunk - 1) / chunk : 1;
    return align_up((size_t)nchunks * (size_t)(nq > 0 ? nq : 1) * K * 8, 256);
}

int qv_bq_scan(const uint64_t* codes, int64_t n, int d, const uint64_t* qcodes, int64_t nq, int K, uint32_t* ids,
               uint32_t* dist, void* workspace, size_t workspace_bytes, void* stream) {
    return qv_bq_scan_enc(codes, n, d, QV_ENC_SM, qcodes, nq, K, ids, dist, workspace, workspace_bytes, stream);
}

int qv_bq_scan_enc(const uint64_t* codes, int64_t n, int d, int encoding, const uint64_t* qcodes, int64_t nq, int K,
                   uint32_t* ids, uint32_t* dist, void* workspace, size_t workspace_bytes, void* stream) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (n < 0 || n >= 0xFFFFFFFFll || nq < 0 || nq > 64ll * 0x7FFFFFFF || K < 1 || K > QV_MAX_SCAN_K || !enc_ok(encoding))
        return QV_ERR_INVALID_ARG;
    if (nq == 0) return QV_OK;
    if ((n > 0 && !codes) || !qcodes || !ids || !dist) return QV_ERR_NULL;
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < qv_bq_scan_workspace_bytes(n, nq, K))
        return QV_ERR_WORKSPACE;
    hipError_t e = qv::launch_bq_scan(codes, n, d, encoding, qcodes, nq, K, static_cast<uint64_t*>(workspace), ids, dist,
                                      (hipStream_t)stream);
    return e == hipSuccess ? QV_OK : hip_fail(e, "code scan launch");
}

int qv_topk_overlap(const uint32_t* a, const uint32_t* b, int64_t nq, int K, uint32_t* hits, void* stream) {
    if (nq < 0 || K < 1) return QV_ERR_INVALID_ARG;
    if (nq == 0) return QV_OK;
    if (!a || !b || !hits) return QV_ERR_NULL;
    hipError_t e = qv::launch_topk_overlap(a, b, nq, K, hits, (hipStream_t)stream);
    return e == hipSuccess ? QV_OK : hip_fail(e, "overlap launch");
}

static bool build_args_ok(int64_t n, int d, int R, int L) {
    return n >= 1 && n < 0xFFFFFFFFll && R >= 1 && R <= 64 && L >= 1 && L <= 192 && d >= 1 && d <= QV_MAX_DIM;
}
// one workgroup per selected edge of a batch: the largest batch, min(max(1, n / 50), max_batch) nodes, times R has to fit a grid
static bool build_batch_ok(int64_t n, int R, int64_t max_batch) {
    if (max_batch < 1) return false;
    int64_t mb = n / 50 < 1 ? 1 : n / 50;
    if (mb > max_batch) mb = max_batch;
    return mb * R <= 0x7FFFFFFFll;
}

size_t qv_build_workspace_bytes(int64_t n, int d, int R, int L, int64_t max_batch) {
    return qv_build_workspace_bytes_enc(n, d, QV_ENC_SM, R, L, max_batch);
}

size_t qv_build_workspace_bytes_enc(int64_t n, int d, int encoding, int R, int L, int64_t max_batch) {
    if (!build_args_ok(n, d, R, L) || !build_batch_ok(n, R, max_batch) || !enc_ok(encoding)) return 0;
    if (qv::build_width_at_least((d + 63) / 64, encoding) == 0) return 0;
    return qv::build_workspace_bytes(n, (d + 63) / 64, encoding, R, L, max_batch);
}

int qv_build_graph(const uint64_t* codes, int64_t n, int d, int R, int L, double alpha, uint32_t entry,
                   int64_t max_batch, uint32_t* adj, void* workspace, size_t workspace_bytes, void* stream) {
    return qv_build_graph_enc(codes, n, d, QV_ENC_SM, R, L, alpha, entry, max_batch, adj, workspace, workspace_bytes, stream);
}

int qv_build_graph_enc(const uint64_t* codes, int64_t n, int d, int encoding, int R, int L, double alpha, uint32_t entry,
                       int64_t max_batch, uint32_t* adj, void* workspace, size_t workspace_bytes, void* stream) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (!build_args_ok(n, d, R, L) || !build_batch_ok(n, R, max_batch) || !(alpha >= 1.0) || (int64_t)entry >= n || !enc_ok(encoding))
        return QV_ERR_INVALID_ARG;
    if (qv::build_width_at_least((d + 63) / 64, encoding) == 0) return QV_ERR_UNSUPPORTED;
    if (!codes || !adj) return QV_ERR_NULL;
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < qv::build_workspace_bytes(n, (d + 63) / 64, encoding, R, L, max_batch))
        return QV_ERR_WORKSPACE;
    hipError_t e = qv::build_graph(codes, n, d, encoding, R, L, alpha, entry, max_batch, adj, workspace, (hipStream_t)stream);
    return e == hipSuccess ? QV_OK : hip_fail(e, "graph construction");
}

int qv_index_load(qv_index** out, int64_t n, int d, int R, const uint32_t* adj, const uint64_t* codes,
                  const float* vecs, uint32_t entry) {
    if (!out) return QV_ERR_NULL;
    *out = nullptr;
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (n < 1 || n >= 0xFFFFFFFFll || R < 1 || R > QV_MAX_DEGREE || (int64_t)entry >= n) return QV_ERR_INVALID_ARG;
    if (!adj || !codes || !vecs) return QV_ERR_NULL;
    qv_index* ix = new (std::nothrow) qv_index;
    if (!ix) return QV_ERR_NOMEM;
    ix->n = n; ix->d = d; ix->R = R; ix->adj = adj; ix->codes = codes; ix->vecs = vecs; ix->entry = entry;
    ix->visited_slots = 0; ix->lanes_per_row = 0; ix->table_format = 0; ix->visited_mode = 0; ix->rerank_mode = 0; ix->encoding = QV_ENC_SM; ix->code_plane_words = 0; ix->code_stride = 0; ix->split1 = ix->split2 = nullptr; ix->timer = nullptr;
    // where the cold data lives decides whether Stage 2 may run inside the search kernel (host memory: never)
    hipPointerAttribute_t attr;
    ix->vecs_on_device = true;
    if (hipPointerGetAttributes(&attr, vecs) == hipSuccess) ix->vecs_on_device = attr.type != hipMemoryTypeHost;
    else (void)hipGetLastError();   // an address the runtime does not know: treat as device memory
    *out = ix;
    return QV_OK;
}

void qv_index_free(qv_index* index) { delete index; }

int qv_index_set_tuning(qv_index* index, int visited_slots, int lanes_per_row, int table_format, int visited_mode,
                        int rerank_mode) {
    if (!index) return QV_ERR_NULL;
    if (visited_slots != 0 && (visited_slots < 1024 || visited_slots > 28672)) return QV_ERR_INVALID_ARG;
    if (table_format != 0 && table_format != 32) return QV_ERR_INVALID_ARG;
    if (visited_mode != 0 && visited_mode != QV_VISITED_EXACT && visited_mode != QV_VISITED_CACHE) return QV_ERR_INVALID_ARG;
    if (rerank_mode != 0 && rerank_mode != QV_RERANK_SEPARATE && rerank_mode != QV_RERANK_FUSED && rerank_mode != QV_RERANK_TAIL) return QV_ERR_INVALID_ARG;
    if (lanes_per_row > 0 && (lanes_per_row > 16 || (lanes_per_row & (lanes_per_row - 1)))) return QV_ERR_INVALID_ARG;
    index->visited_slots = visited_slots;
    index->lanes_per_row = lanes_per_row;
    index->table_format = table_format;
    index->visited_mode = visited_mode;
    index->rerank_mode = rerank_mode;
    return QV_OK;
}

int qv_index_set_encoding(qv_index* index, int encoding) {
    if (!index) return QV_ERR_NULL;
    if (!enc_ok(encoding)) return QV_ERR_INVALID_ARG;
    index->encoding = encoding;
    return QV_OK;
}

// lines of 128 bytes a row of `bytes` bytes touches on average when rows are `bytes` apart (dense) ...
static double dense_lines(int bytes) {
    int g = bytes, r = 128;
    while (r) { int t = g % r; g = r; r = t; }      // rows start at every multiple of gcd(bytes, 128) within a line
    return (bytes + 128 - g) / 128.0;
}

int qv_code_layout(int d, int encoding, int* plane_words, int* stride) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (!enc_ok(encoding)) return QV_ERR_INVALID_ARG;
    if (!plane_words || !stride) return QV_ERR_NULL;
    const int nw = (d + 63) / 64, planes = encoding == QV_ENC_SIGN1 ? 1 : 2;
    // planes as wide as the nearest width the search kernel is compiled for, if that costs at most a third more
    int pw = qv::search_compiled_width_at_least(nw, encoding);
    if (pw == 0 || 3 * pw > 4 * nw || pw > max_plane_words(nw)) pw = nw;
    const int bytes = planes * pw * 8;
    // smallest stride >= the row that divides 128 bytes or is a multiple of them, if rows then touch fewer lines
    const int padded = bytes <= 16 ? 16 : (bytes <= 32 ? 32 : (bytes <= 64 ? 64 : (bytes + 127) / 128 * 128));
    const double padded_lines = padded <= 128 ? 1.0 : padded / 128.0;
    *plane_words = pw;
    *stride = padded_lines < dense_lines(bytes) ? padded / 8 : planes * pw;
    return QV_OK;
}

static bool layout_ok(int d, int encoding, int plane_words, int stride) {
    const int nw = (d + 63) / 64, planes = encoding == QV_ENC_SIGN1 ? 1 : 2;
    if (plane_words < nw || plane_words > max_plane_words(nw)) return false;
    const int row = planes * plane_words;
    return stride == row || (stride > row && !(stride & 1) && stride <= 4 * row + 16);
}

int qv_pad_codes(const uint64_t* codes, int64_t n, int d, int encoding, int plane_words, int stride, uint64_t* out,
                 void* stream) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (!enc_ok(encoding) || n < 0 || !layout_ok(d, encoding, plane_words, stride)) return QV_ERR_INVALID_ARG;
    if (n == 0) return QV_OK;
    if (!codes || !out) return QV_ERR_NULL;
    hipError_t e = qv::launch_pad_codes(codes, n, (d + 63) / 64, encoding == QV_ENC_SIGN1 ? 1 : 2, plane_words, stride, out,
                                        (hipStream_t)stream);
    return e == hipSuccess ? QV_OK : hip_fail(e, "code padding launch");
}

int qv_index_set_code_layout(qv_index* index, int plane_words, int stride) {
    if (!index) return QV_ERR_NULL;
    if (plane_words == 0 && stride == 0) {   // back to dense rows
        index->code_plane_words = index->code_stride = 0;
        return QV_OK;
    }
    if (!layout_ok(index->d, index->encoding, plane_words, stride)) return QV_ERR_INVALID_ARG;
    index->code_plane_words = plane_words;
    index->code_stride = stride;
    return QV_OK;
}

int qv_split_layout(int d, int* words1, int* words2) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (!words1 || !words2) return QV_ERR_NULL;
    const int nw = (d + 63) / 64;
    if (qv::split_lanes_per_row(nw) == 0) return QV_ERR_UNSUPPORTED;
    *words1 = qv::split_stride1(nw);
    *words2 = qv::split_stride2(nw);
    return QV_OK;
}

int qv_split_codes(const uint64_t* codes, int64_t n, int d, uint64_t* out1, uint64_t* out2, void* stream) {
    if (d < 1 || d > QV_MAX_DIM) return QV_ERR_DIM;
    if (n < 0) return QV_ERR_INVALID_ARG;
    const int nw = (d + 63) / 64;
    if (qv::split_lanes_per_row(nw) == 0) return QV_ERR_UNSUPPORTED;
    if (n == 0) return QV_OK;
    if (!codes || !out1 || !out2) return QV_ERR_NULL;
    hipError_t e = qv::launch_split_codes(codes, n, nw, out1, out2, (hipStream_t)stream);
    return e == hipSuccess ? QV_OK : hip_fail(e, "code split launch");
}

int qv_index_set_split_codes(qv_index* index, const uint64_t* split1, const uint64_t* split2) {
    if (!index) return QV_ERR_NULL;
    if (!split1 && !split2) {   // back to the rows given at load time
        index->split1 = index->split2 = nullptr;
        return QV_OK;
    }
    if (!split1 || !split2) return QV_ERR_NULL;
    if (index->encoding != QV_ENC_SM || qv::split_lanes_per_row((index->d + 63) / 64) == 0) return QV_ERR_UNSUPPORTED;
    if (((uintptr_t)split1 & 127u) || ((uintptr_t)split2 & 15u)) return QV_ERR_INVALID_ARG;
    index->split1 = split1;
    index->split2 = split2;
    return QV_OK;
}

// Where Stage 2 runs for this beam width: QV_RERANK_SEPARATE, QV_RERANK_FUSED or QV_RERANK_TAIL (see quiver.h).
static int rerank_place(const qv_index* index, int ef) {
    const bool in_kernel_ok = ef <= 128 && index->vecs_on_device;
    if (!in_kernel_ok || index->rerank_mode == QV_RERANK_SEPARATE) return QV_RERANK_SEPARATE;
    return index->rerank_mode != 0 ? index->rerank_mode : QV_RERANK_TAIL;
}

int qv_index_rerank_fused(const qv_index* index, int ef) {
    if (!index) return QV_ERR_NULL;
    return rerank_place(index, ef) != QV_RERANK_SEPARATE ? 1 : 0;
}

size_t qv_search_workspace_bytes(int64_t nq, int d, int k, int ef) {
    if (nq < 0 || d < 1 || d > QV_MAX_DIM || ef < 1 || ef > QV_MAX_EF || k < 1 || k > ef) return 0;
    return layout(nq > 0 ? nq : 1, d, ef).total;
}

// ---------------------------------------------------------------------------------------------
// Scratch of qv_search_static: one array per GPU, part of the loaded code object, never allocated or freed.  In host
// code its name is only a handle for hipGetSymbolAddress; the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[QV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// device address of `scratch` on the current device; QV_OK or an error
int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return QV_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!ptr) return hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch) gave no address");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return QV_OK;
}
}  // namespace

int qv_search_static(const qv_index* index, const float* queries, int64_t nq, int k, int ef, uint32_t* ids,
                     float* scores, const qv_trace* trace, void* stream) {
    if (!index) return QV_ERR_NULL;
    if (nq < 0 || nq > 0x7FFFFFFFll || k < 1) return QV_ERR_INVALID_ARG;
    if (ef < 1 || ef > QV_MAX_EF) return QV_ERR_EF_RANGE;
    if (k > ef) return QV_ERR_EF_LT_K;
    if (nq == 0) return QV_OK;
    if (layout(nq, index->d, ef).total > (size_t)QV_STATIC_SCRATCH_BYTES) return QV_ERR_SCRATCH_LIMIT;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != QV_OK) return rc;
    return qv_search(index, queries, nq, k, ef, ids, scores, ws, QV_STATIC_SCRATCH_BYTES, trace, stream);
}

int qv_search(const qv_index* index, const float* queries, int64_t nq, int k, int ef, uint32_t* ids, float* scores,
              void* workspace, size_t workspace_bytes, const qv_trace* trace, void* stream_) {
    if (!index) return QV_ERR_NULL;
    if (nq < 0 || nq > 0x7FFFFFFFll || k < 1) return QV_ERR_INVALID_ARG;
    if (ef < 1 || ef > QV_MAX_EF) return QV_ERR_EF_RANGE;
    if (k > ef) return QV_ERR_EF_LT_K;
    if (trace && trace->visit_order && trace->visit_cap < 1) return QV_ERR_INVALID_ARG;
    if (nq == 0) return QV_OK;
    if (!queries || !ids || !scores) return QV_ERR_NULL;
    const WorkspaceLayout L = layout(nq, index->d, ef);
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < L.total) return QV_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = static_cast<char*>(workspace);
    uint64_t* qcodes = reinterpret_cast<uint64_t*>(ws + L.qcodes);

    const int nw = (index->d + 63) / 64, planes = index->encoding == QV_ENC_SIGN1 ? 1 : 2;
    int plane_words = nw, row_stride = planes * nw;
    if (index->code_stride > 0) {
        if (!layout_ok(index->d, index->encoding, index->code_plane_words, index->code_stride))
            return QV_ERR_INVALID_ARG;  // the layout was set before the encoding changed
        plane_words = index->code_plane_words;
        row_stride = index->code_stride;
    }

    qv_timer* tm = index->timer;
    hipEvent_t* ev = nullptr;
    if (tm && tm->used < tm->max_calls) ev = tm->ev + 4 * (size_t)tm->used++;
    hipError_t e;
    if (ev && (e = hipEventRecord(ev[0], stream)) != hipSuccess) return hip_fail(e, "event record");

    // Stage 1 preamble: the query's own code, then (index stored with wider planes) the same words in that layout
    // (a query that holds Inf or NaN is flagged here and not searched: see the kernel)
    uint32_t* qstatus = reinterpret_cast<uint32_t*>(ws + L.qstatus);
    e = qv::launch_encode(queries, nq, index->d, index->encoding, qcodes, qstatus, stream);
    if (e != hipSuccess) return hip_fail(e, "query encode launch");
    if (plane_words != nw) {
        uint64_t* wide = reinterpret_cast<uint64_t*>(ws + L.qcodes_wide);
        e = qv::launch_pad_codes(qcodes, nq, nw, planes, plane_words, planes * plane_words, wide, stream);
        if (e != hipSuccess) return hip_fail(e, "query code layout launch");
        qcodes = wide;
    }

    qv::SearchParams sp;
    sp.adj = index->adj; sp.codes = index->codes; sp.qcodes = qcodes; sp.encoding = index->encoding;
    sp.row_stride = row_stride; sp.qstatus = qstatus;
    // rows in the split layout are read by the search kernel only; they hold planes of ceil(d/64) words
    const bool split = index->split1 && index->encoding == QV_ENC_SM && plane_words == nw;
    sp.codes1 = split ? index->split1 : nullptr; sp.codes2 = split ? index->split2 : nullptr;
    sp.n = index->n; sp.nq = nq; sp.nw = plane_words; sp.R = index->R; sp.entry = index->entry; sp.ef = ef;
    // Visited set.  Default: a cache of 4096 slots (8 KB of 16-bit tags): with the list and the merge area a
    // query then needs about 10 KB of LDS, so 16 queries fit a compute unit and registers, not LDS, bound the
    // occupancy; at the beam widths of interest it forgets few ids (about 1 % more distance evaluations at
    // ef = 64).  QV_VISITED_EXACT: about two slots per expected distance evaluation (~45 per unit of ef at
    // degree 64), as far as 64 KB of LDS per query allow.
    const bool cache = index->visited_mode != QV_VISITED_EXACT;
    // (wider beams: the merge area grows to 8.7 KB at ef = 1024, so the cache shrinks to keep the queries per CU up;
    // measured optima at 1M x 768: 3072 slots for ef 129..512, 2048 beyond -- ef = 1024: 26.2 / 25.1 / 28.4 / 27.7 ms
    // per 10,000 queries with 1024 / 2048 / 3072 / 4096 slots, 74 / 61 / 52 / 45 % of the nodes evaluated again)
    // (short rows, planes of up to 6 words: the kernel needs few enough registers for a fifth wave per SIMD, which a
    // 3072-slot cache lets LDS hold: 1M x 384, ef = 64: 1.00 -> 0.98 ms per batch at 1 % more evaluations)
    const int cache_slots = ef <= 128 ? (plane_words <= 6 ? 3072 : 4096) : (ef <= 512 ? 3072 : 2048);
    int slots = index->visited_slots > 0 ? index->visited_slots : (cache ? cache_slots : 96 * ef + 2048);
    const size_t fixed = qv::beam_search_lds_bytes(sp.nw, 0, true, ef);
    const int max_narrow = (int)((65536 - fixed) / 2 / 1024 * 1024);
    if (slots > max_narrow) slots = max_narrow;
    if (slots < 1024) slots = 1024;
    qv::plan_visited_table(sp, (uint32_t)slots, index->table_format != 32, cache);
    if (sp.vis_regions == 0 && sp.vis_slots > 8192) {  // 32-bit entries: keep the table within 32 KB of LDS
        qv::plan_visited_table(sp, 8192, false, cache);
    }
    // Stage 2 inside the search launch (beams of up to 128 entries over vectors in device memory), by default by other
    // waves of the launch that start when the last searches are under way (QV_RERANK_TAIL).  Measured per 10,000
    // queries, ef = 64, kernel of its own / by the searching wave / by other waves: 1M x 384: 1.21 / 1.16 / 1.12 ms,
    // 1M x 512: 1.27 / 1.22 / 1.19, 1M x 768: 1.24 / 1.33 / 1.23, 5M x 1024: 2.12 / - / 2.10, 1M x 3072: 4.63 / 4.92 /
    // 4.37.  Inside the launch, the final lists leave it only if the caller's trace asks for them or other waves need
    // them.
    int place = rerank_place(index, ef);
    if (place == QV_RERANK_TAIL && nq > (1ll << 30)) place = QV_RERANK_FUSED;   // two workgroups per query must fit a grid
    const bool fused = place != QV_RERANK_SEPARATE, tail = place == QV_RERANK_TAIL;
    // the final lists go straight into the caller's trace buffers when there are any
    sp.cand_ids = trace && trace->cand_ids ? trace->cand_ids : reinterpret_cast<uint32_t*>(ws + L.cand_ids);
    sp.cand_dist = trace && trace->cand_dist ? trace->cand_dist : reinterpret_cast<uint32_t*>(ws + L.cand_dist);
    sp.n_cand = trace && trace->n_cand ? trace->n_cand : reinterpret_cast<uint32_t*>(ws + L.n_cand);
    if (fused && !tail && !(trace && (trace->cand_ids || trace->cand_dist))) sp.cand_ids = sp.cand_dist = nullptr;
    if (fused && !tail && !(trace && trace->n_cand)) sp.n_cand = nullptr;
    sp.n_expanded = trace ? trace->n_expanded : nullptr;
    sp.n_evals = trace ? trace->n_dist_evals : nullptr;
    sp.status = trace ? trace->status : nullptr;
    sp.visit_order = trace ? trace->visit_order : nullptr;
    sp.visit_cap = trace && trace->visit_order ? trace->visit_cap : 0;
    sp.rr_queries = fused ? queries : nullptr; sp.rr_vecs = fused ? index->vecs : nullptr;
    sp.rr_d = index->d; sp.rr_k = k; sp.rr_ids = ids; sp.rr_scores = scores;
    sp.rr_ticket = tail ? reinterpret_cast<uint32_t*>(ws + L.rr_ticket) : nullptr;
    sp.rr_done = tail ? reinterpret_cast<uint32_t*>(ws + L.rr_done) : nullptr;
    sp.rr_spin_limit = 1u << 22;   // about seven seconds; a search takes milliseconds
    sp.order = nullptr;
    if (qv::launch_query_order(sp, reinterpret_cast<uint32_t*>(ws + L.order), sp.rr_ticket, sp.rr_done, stream, &e))
        sp.order = reinterpret_cast<uint32_t*>(ws + L.order);
    if (e != hipSuccess) return hip_fail(e, "query order launch");
    if (ev && (e = hipEventRecord(ev[1], stream)) != hipSuccess) return hip_fail(e, "event record");
    e = qv::launch_beam_search(sp, index->lanes_per_row, stream);
    if (e != hipSuccess) return hip_fail(e, "beam search launch");
    if (ev && (e = hipEventRecord(ev[2], stream)) != hipSuccess) return hip_fail(e, "event record");

    if (!fused) {
        qv::RerankParams rp;
        rp.queries = queries; rp.vecs = index->vecs; rp.cand_ids = sp.cand_ids; rp.n_cand = sp.n_cand;
        rp.nq = nq; rp.d = index->d; rp.ef = ef; rp.k = k; rp.ids = ids; rp.scores = scores;
        e = qv::launch_rerank(rp, stream);
        if (e != hipSuccess) return hip_fail(e, "rerank launch");
    }
    if (ev && (e = hipEventRecord(ev[3], stream)) != hipSuccess) return hip_fail(e, "event record");

    return QV_OK;
}

int qv_timer_create(qv_timer** out, int max_calls) {
    if (!out) return QV_ERR_NULL;
    *out = nullptr;
    if (max_calls < 1 || max_calls > 65536) return QV_ERR_INVALID_ARG;
    qv_timer* t = new (std::nothrow) qv_timer;
    if (!t) return QV_ERR_NOMEM;
    t->max_calls = max_calls; t->used = 0;
    t->ev = new (std::nothrow) hipEvent_t[4 * (size_t)max_calls];
    if (!t->ev) { delete t; return QV_ERR_NOMEM; }
    for (int i = 0; i < 4 * max_calls; ++i) {
        hipError_t e = hipEventCreate(&t->ev[i]);
        if (e != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(t->ev[j]);
            delete[] t->ev; delete t;
            return hip_fail(e, "event create");
        }
    }
    *out = t;
    return QV_OK;
}

void qv_timer_free(qv_timer* t) {
    if (!t) return;
    for (int i = 0; i < 4 * t->max_calls; ++i) (void)hipEventDestroy(t->ev[i]);
    delete[] t->ev;
    delete t;
}

void qv_index_set_timer(qv_index* index, qv_timer* t) { if (index) index->timer = t; }

int qv_timer_read(qv_timer* t, float* ms, int max_calls) {
    if (!t || !ms) return QV_ERR_NULL;
    int n = t->used < max_calls ? t->used : max_calls;
    for (int c = 0; c < n; ++c) {
        hipEvent_t* ev = t->ev + 4 * (size_t)c;
        hipError_t e = hipEventSynchronize(ev[3]);
        if (e != hipSuccess) return hip_fail(e, "event synchronize");
        for (int s = 0; s < 3; ++s) {
            e = hipEventElapsedTime(&ms[3 * c + s], ev[s], ev[s + 1]);
            if (e != hipSuccess) return hip_fail(e, "event elapsed");
        }
    }
    t->used = 0;
    return n;
}

const char* qv_strerror(int code) {
    switch (code) {
        case QV_OK: return "ok";
        case QV_ERR_INVALID_ARG: return "a size or count is out of range";
        case QV_ERR_NULL: return "a required pointer is NULL";
        case QV_ERR_DIM: return "dimension out of range";
        case QV_ERR_EF_LT_K: return "k is larger than ef";
        case QV_ERR_EF_RANGE: return "ef out of range";
        case QV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case QV_ERR_HIP: return "HIP runtime error";
        case QV_ERR_NOMEM: return "host allocation failed";
        case QV_ERR_UNSUPPORTED: return "shape not supported by this entry point";
        case QV_ERR_SCRATCH_LIMIT: return "the batch needs more scratch than the library's built-in buffer holds (QV_STATIC_SCRATCH_BYTES)";
        default: return "unknown error code";
    }
}

const char* qv_last_hip_error(void) { return g_hip_error; }

}  // extern "C"
