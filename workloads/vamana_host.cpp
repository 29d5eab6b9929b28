// Host-side generator of the navigation graph that both the CPU oracle and the GPU library
// consume as an INPUT (the paper's Sec. 3.2, Algorithm 1 "BQ-Vamana Edge Selection" with
// bidirectional re-selection, Sec. 2.2; R = 2m, L = ef_c, alpha as in Sec. 5.1).
//
// This is workload-generation support code, not the product and not the oracle: it has its
// own quick encoder and its own popcount distance, shares no code with either, and any
// adjacency it emits is a valid input (its quality moves recall, never parity).
//
// Construction is batch-synchronous instead of the paper's lock-based concurrent insertion
// (Sec. 4.1): nodes are inserted in id order in batches; all nodes of a batch search the graph
// as it stood before the batch, select their out-edges, and then every touched target merges
// its new in-edges, re-running the edge selection when it would exceed R.  The result does not
// depend on the number of threads.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <thread>
#include <vector>

static const uint32_t EMPTY = 0xFFFFFFFFu;

#ifndef VH_VARIANT_ONLY
#define VH_NS vh_generic
#include "vamana_core.inc"
#undef VH_NS

// the popcount-heavy variant lives in a second object file compiled with AVX-512 VPOPCNTDQ
namespace vh_avx512 {
int build(const uint64_t*, int64_t, int, int, int, double, uint32_t, uint32_t*, int, const char*, double, int64_t);
uint32_t nearest_code(const uint64_t*, int64_t, int, const uint64_t*, int);
}  // namespace vh_avx512

static bool have_avx512() {
    return __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512vl") &&
           __builtin_cpu_supports("avx512bw") && __builtin_cpu_supports("avx512vpopcntdq");
}

static void quick_encode(const float* x, int d, uint64_t* code) {
    int W = (d + 63) / 64;
    double s = 0;
    for (int i = 0; i < d; ++i) s += std::fabs((double)x[i]);
    for (int w = 0; w < 2 * W; ++w) code[w] = 0;
    for (int i = 0; i < d; ++i) {
        if (x[i] > 0) code[i / 64] |= 1ull << (i % 64);
        if (std::fabs((double)x[i]) * d > s) code[W + i / 64] |= 1ull << (i % 64);
    }
}

extern "C" {

int vh_uses_avx512() { return have_avx512() ? 1 : 0; }

// x[n][d] -> codes[n][2*ceil(d/64)] with a plain double-precision mean (not the exact one)
int vh_encode(const float* x, int64_t n, int d, uint64_t* codes, int threads) {
    if (!x || !codes || n < 0 || d < 1) return -1;
    int cw = 2 * ((d + 63) / 64);
    vh_generic::parallel_for(n, threads, [&](int64_t v, int) { quick_encode(x + (size_t)v * d, d, codes + (size_t)v * cw); });
    return 0;
}

// entry = node whose code is nearest to the code of the float32 centroid (ties: smallest id)
int64_t vh_pick_entry(const float* x, const uint64_t* codes, int64_t n, int d, int threads) {
    if (!x || !codes || n < 1 || d < 1) return -1;
    std::vector<double> c((size_t)d, 0.0);
    for (int64_t v = 0; v < n; ++v)
        for (int i = 0; i < d; ++i) c[(size_t)i] += x[(size_t)v * d + i];
    std::vector<float> cf((size_t)d);
    for (int i = 0; i < d; ++i) cf[(size_t)i] = (float)(c[(size_t)i] / (double)n);
    int W = (d + 63) / 64;
    std::vector<uint64_t> cc((size_t)2 * W);
    quick_encode(cf.data(), d, cc.data());
    return have_avx512() ? vh_avx512::nearest_code(codes, n, W, cc.data(), threads)
                         : vh_generic::nearest_code(codes, n, W, cc.data(), threads);
}

// adj[n][R] (0xFFFFFFFF = empty slot) is written in full
int vh_build(const uint64_t* codes, int64_t n, int d, int R, int L, double alpha, uint32_t entry, uint32_t* adj,
             int threads, const char* progress_path, double batch_frac, int64_t max_batch) {
    if (!codes || !adj || n < 1 || n >= 0xFFFFFFFFll || d < 1 || R < 1 || R > 1024 || L < 1 || alpha < 1.0 ||
        entry >= n)
        return -1;
    if (batch_frac <= 0) batch_frac = 0.02;
    if (max_batch < 1) max_batch = 1 << 20;
    int W = (d + 63) / 64;
    return have_avx512()
               ? vh_avx512::build(codes, n, W, R, L, alpha, entry, adj, threads, progress_path, batch_frac, max_batch)
               : vh_generic::build(codes, n, W, R, L, alpha, entry, adj, threads, progress_path, batch_frac, max_batch);
}

}  // extern "C"

#else  // VH_VARIANT_ONLY: the AVX-512 object

#define VH_NS vh_avx512_impl
#include "vamana_core.inc"
#undef VH_NS
namespace vh_avx512 {
int build(const uint64_t* codes, int64_t n, int W, int R, int L, double alpha, uint32_t entry, uint32_t* adj,
          int threads, const char* progress_path, double batch_frac, int64_t max_batch) {
    return vh_avx512_impl::build(codes, n, W, R, L, alpha, entry, adj, threads, progress_path, batch_frac, max_batch);
}
uint32_t nearest_code(const uint64_t* codes, int64_t n, int W, const uint64_t* target, int threads) {
    return vh_avx512_impl::nearest_code(codes, n, W, target, threads);
}
}  // namespace vh_avx512

#endif
