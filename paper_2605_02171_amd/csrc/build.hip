// Graph construction in code space on the GPU (paper Sec. 3.2, Algorithm 1 "BQ-Vamana Edge Selection",
// with the bidirectional re-selection of Sec. 2.2), batch-synchronous reading:
//   nodes are inserted in id order in batches of max(1, done/50); every node of a batch searches the
//   graph as it stood before the batch (beam width L, the library's own beam-search kernel), takes as
//   candidates its final list plus its current out-neighbours and selects its out-edges by Algorithm 1;
//   then every selected node b receives the selecting nodes as in-edge candidates (at most the 192
//   nearest per batch): added if they fit in the row, otherwise the row is re-selected by Algorithm 1
//   from (old row U new candidates).
// The paper's own construction is lock-based and concurrent (Sec. 4.1) and has no single defined
// result; this reading is a function of its inputs, so it can be checked bit for bit.
//
// Per batch: beam_search_kernel -> forward_select_kernel (one wave per new node; every selected edge (target,
// source) also counts itself in at its target and learns its rank there) -> reserve_segments_kernel (the edge of
// rank 0 reserves a segment of the source array for its target) -> scatter_sources_kernel (every edge puts its
// source at segment start + rank) -> reverse_kernel (one wave per target, started by the edge of rank 0).
// Grouping the edges by target this way takes three atomics per edge and no sort; the order of the segments and
// inside them depends on the order of the atomics, the result does not (the reverse step ranks its candidates
// by (distance, id) itself).  Algorithm 1 runs with one lane per already selected neighbour: the candidate's
// code is wave-uniform (scalar loads), every lane keeps "its" selected code in registers and computes one
// distance, a ballot decides.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace qv {

constexpr uint64_t B_NONE = ~0ull;
constexpr int BUF = 256;       // candidate keys (dist << 32 | id) a wave can sort
constexpr int MAX_NEW = 192;   // new in-edge candidates a node considers per batch
constexpr int N_BUCKETS = 1024;

__device__ __forceinline__ void bsync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// ascending bitonic sort of buf[0..m), m in {64, 128, 256}, by one wave
__device__ void sort_keys(uint64_t* buf, int m, int lane) {
    for (int k = 2; k <= m; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int pp = lane; pp < (m >> 1); pp += 64) {
                const int i = ((pp & ~(j - 1)) << 1) | (pp & (j - 1));
                const int l = i | j;
                const uint64_t a = buf[i], b = buf[l];
                const bool up = (i & k) == 0;
                if ((a > b) == up) { buf[i] = b; buf[l] = a; }
            }
            bsync();
        }
    }
}

__device__ __forceinline__ int pow2_at_least(int c) { return c <= 64 ? 64 : (c <= 128 ? 128 : 256); }

// one 32-bit step of the distance between two codes (a0, a1 / b0, b1: first and second plane dword of each) under
// the three encodings: Sign-Magnitude (Table 1 as three popcounts), 1-bit sign (Hamming), 2-bit uniform quantiser
// (L1 on levels = Hamming distance of the three thermometer planes hi|lo, hi, hi&lo)
template <int ENC>
__device__ __forceinline__ void pair_accumulate(uint32_t a0, uint32_t a1, uint32_t b0, uint32_t b1, uint32_t& c1,
                                                uint32_t& c2, uint32_t& c3) {
    if constexpr (ENC == ENC_SM) {
        const uint32_t x = a0 ^ b0;
        c1 += __popc(x);
        c2 += __popc(__builtin_amdgcn_bitop3_b32(x, a1, b1, 0xE0));
        c3 += __popc(__builtin_amdgcn_bitop3_b32(x, a1, b1, 0x80));
    } else if constexpr (ENC == ENC_SIGN1) {
        c1 += __popc(a0 ^ b0);
    } else {
        c1 += __popc(__builtin_amdgcn_bitop3_b32(a1, a0, b0 | b1, 0x56));
        c2 += __popc(a1 ^ b1);
        c3 += __popc(__builtin_amdgcn_bitop3_b32(a1, a0, b0 & b1, 0x6A));
    }
}
template <int ENC>
__device__ __forceinline__ uint32_t pair_distance(uint32_t c1, uint32_t c2, uint32_t c3) {
    return ENC == ENC_SM ? c1 + c2 + 2u * c3 : c1 + c2 + c3;
}

// distance between a wave-uniform code (scalar pointer) and a per-lane code in memory
template <int ENC, int NW_T>
__device__ __forceinline__ uint32_t dist_uniform_vs_row(const uint32_t* __restrict__ cu, const uint64_t* __restrict__ codes,
                                                        uint32_t v) {
    constexpr int DW = 2 * NW_T, PLANES = ENC == ENC_SIGN1 ? 1 : 2;
    const uint32_t* r = reinterpret_cast<const uint32_t*>(codes + (int64_t)v * (PLANES * NW_T));
    uint32_t c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
    for (int w = 0; w < DW; ++w)
        pair_accumulate<ENC>(r[w], PLANES == 2 ? r[DW + w] : 0u, cu[w], PLANES == 2 ? cu[DW + w] : 0u, c1, c2, c3);
    return pair_distance<ENC>(c1, c2, c3);
}

// Algorithm 1 over buf[0..count) (sorted ascending, ids distinct, self excluded).  sel[0..ns) receives the ids.
template <int ENC, int NW_T>
__device__ int select_edges_dev(const uint64_t* __restrict__ codes, const uint64_t* buf, int count, int R, double alpha,
                                uint32_t* sel, int lane) {
    constexpr int DW = 2 * NW_T, PLANES = ENC == ENC_SIGN1 ? 1 : 2;
    uint32_t sc[PLANES * DW];  // the code of the neighbour this lane stands for
#pragma unroll
    for (int w = 0; w < PLANES * DW; ++w) sc[w] = 0;
    int ns = 0;
    for (int i = 0; i < count; ++i) {
        const uint64_t key = buf[i];
        const uint32_t c = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)key);
        const uint32_t dct = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(key >> 32));
        const uint32_t* crow = reinterpret_cast<const uint32_t*>(codes + (int64_t)c * (PLANES * NW_T));  // wave-uniform
        uint32_t c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
        for (int w = 0; w < DW; ++w)
            pair_accumulate<ENC>(sc[w], PLANES == 2 ? sc[DW + w] : 0u, crow[w], PLANES == 2 ? crow[DW + w] : 0u, c1, c2, c3);
        const uint32_t dcs = pair_distance<ENC>(c1, c2, c3);
        const bool viol = lane < ns && !((double)dct <= alpha * (double)dcs);
        if (!__any(viol)) {
            if (lane == ns) {
#pragma unroll
                for (int w = 0; w < PLANES * DW; ++w) sc[w] = crow[w];
            }
            if (lane == 0) sel[ns] = c;
            ns++;
            if (ns == R) break;
        }
    }
    bsync();
    return ns;
}

struct BuildParams {
    const uint64_t* codes;
    uint32_t* adj;
    int64_t n;
    int R, L;
    double alpha;
    int64_t done, bs;
    const uint32_t* cand_ids;   // [bs][L]
    const uint32_t* cand_dist;  // [bs][L]
    const uint32_t* n_cand;     // [bs]
    // in-edges of the batch, grouped by target (edge e = i * R + j is the j-th edge selected by batch node i)
    uint32_t* edge_target;      // [bs*R] target of edge e, EMPTY_ID where node i selected fewer than j + 1 edges
    uint32_t* edge_rank;        // [bs*R] how many edges had counted themselves in at the same target before e
    uint32_t* tgt_count;        // [n]    edges of this batch per target; 0 outside the reverse step
    uint32_t* tgt_start;        // [n]    where the target's sources start in `sources`
    uint32_t* edge_start;       // [bs*R] for the edge of rank 0 at a target: tgt_start and ...
    uint32_t* edge_count;       // [bs*R] ... tgt_count of that target (what the reverse step needs, next to the edge)
    // order of the reverse step: targets bucketed by id range (N_BUCKETS ranges of 2^bkt_shift ids), so that waves
    // running at the same time work on neighbouring rows of the adjacency and of the codes
    uint32_t* edge_bpos;        // [bs*R] for the edge of rank 0 at a target: its position inside the target's bucket
    uint32_t* bkt_count;        // [N_BUCKETS] targets per bucket; 0 between batches
    uint32_t* bkt_offset;       // [N_BUCKETS + 1] where each bucket starts in owner_list; last entry: number of targets
    uint32_t* owner_list;       // [bs*R] edges of rank 0, bucket by bucket
    int bkt_shift;
    uint32_t* sources;          // [bs*R] sources, one segment per target
    uint32_t* cursor;           // [1]    words of `sources` reserved so far; 0 between batches
};

template <int ENC, int NW_T>
__global__ __launch_bounds__(64) void forward_select_kernel(BuildParams p) {
    __shared__ uint64_t buf[BUF];
    __shared__ uint32_t sel[64];
    const int lane = threadIdx.x;
    const int64_t i = blockIdx.x;
    const uint32_t t = (uint32_t)(p.done + i);
    const int nc = (int)p.n_cand[i];
    int removed = 0;
    for (int e = lane; e < BUF; e += 64) {
        uint64_t key = B_NONE;
        if (e < nc) {
            const uint32_t id = p.cand_ids[i * p.L + e];
            if (id != t) key = ((uint64_t)p.cand_dist[i * p.L + e] << 32) | id;
        }
        buf[e] = key;
        removed += __popcll(__ballot(e < nc && key == B_NONE));
    }
    int total = nc;
    // current out-neighbours (only a node that was reachable before its own turn has any)
    const uint32_t v = lane < p.R ? p.adj[(int64_t)t * p.R + lane] : EMPTY_ID;
    const bool has = v != EMPTY_ID && v != t;
    bsync();
    if (__any(has)) {
        bool dup = false;
        for (int e = 0; e < nc; ++e) dup |= (uint32_t)buf[e] == v;
        const bool add = has && !dup;
        const uint32_t* ct = reinterpret_cast<const uint32_t*>(p.codes + (int64_t)t * ((ENC == ENC_SIGN1 ? 1 : 2) * NW_T));
        const uint32_t dv = add ? dist_uniform_vs_row<ENC, NW_T>(ct, p.codes, v) : 0u;
        const uint64_t am = __ballot(add);
        const int pos = total + __popcll(am & ((1ull << lane) - 1ull));
        if (add && pos < BUF) buf[pos] = ((uint64_t)dv << 32) | v;
        total += __popcll(am);
        bsync();
    }
    sort_keys(buf, pow2_at_least(total), lane);
    const int ns = select_edges_dev<ENC, NW_T>(p.codes, buf, total - removed, p.R, p.alpha, sel, lane);
    if (lane < p.R) {
        const uint32_t s = lane < ns ? sel[lane] : EMPTY_ID;
        p.adj[(int64_t)t * p.R + lane] = s;
        p.edge_target[i * p.R + lane] = s;
        if (lane < ns) p.edge_rank[i * p.R + lane] = atomicAdd(p.tgt_count + s, 1u);
    }
}

// one thread per edge: the first edge that reached a target reserves room for all of that target's sources
__global__ __launch_bounds__(256) void reserve_segments_kernel(BuildParams p, int64_t n_edges) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n_edges) return;
    const uint32_t b = p.edge_target[e];
    if (b == EMPTY_ID || p.edge_rank[e] != 0) return;
    const uint32_t count = p.tgt_count[b], start = atomicAdd(p.cursor, count);
    p.tgt_start[b] = start;
    p.edge_start[e] = start;
    p.edge_count[e] = count;
    p.edge_bpos[e] = atomicAdd(p.bkt_count + min(b >> p.bkt_shift, (uint32_t)(N_BUCKETS - 1)), 1u);
}

// one workgroup: exclusive prefix sum over the bucket counts (which it clears for the next batch)
__global__ __launch_bounds__(N_BUCKETS) void bucket_offsets_kernel(BuildParams p) {
    __shared__ uint32_t sums[N_BUCKETS];
    const int t = threadIdx.x;
    const uint32_t mine = p.bkt_count[t];
    p.bkt_count[t] = 0;
    sums[t] = mine;
    __syncthreads();
    for (int off = 1; off < N_BUCKETS; off <<= 1) {
        const uint32_t add = t >= off ? sums[t - off] : 0u;
        __syncthreads();
        sums[t] += add;
        __syncthreads();
    }
    p.bkt_offset[t] = sums[t] - mine;
    if (t == N_BUCKETS - 1) p.bkt_offset[N_BUCKETS] = sums[t];
}

// one thread per edge: the source (batch node e / R) goes to its place in the target's segment
__global__ __launch_bounds__(256) void scatter_sources_kernel(BuildParams p, int64_t n_edges) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n_edges) return;
    if (e == 0) *p.cursor = 0;                           // every segment is reserved by now; the next batch starts at 0
    const uint32_t b = p.edge_target[e];
    if (b == EMPTY_ID) return;
    const uint32_t rank = p.edge_rank[e];
    p.sources[p.tgt_start[b] + rank] = (uint32_t)(p.done + e / p.R);
    if (rank == 0) p.owner_list[p.bkt_offset[min(b >> p.bkt_shift, (uint32_t)(N_BUCKETS - 1))] + p.edge_bpos[e]] = (uint32_t)e;
}

template <int ENC, int NW_T>
__global__ __launch_bounds__(64) void reverse_kernel(BuildParams p) {
    __shared__ uint64_t buf[BUF];
    __shared__ uint32_t sel[64];
    __shared__ uint32_t rowcopy[64];
    const int lane = threadIdx.x;
    if (blockIdx.x >= p.bkt_offset[N_BUCKETS]) return;   // one workgroup per target of the batch, in bucket order
    const int64_t e0 = p.owner_list[blockIdx.x];         // the edge of rank 0 at that target
    const uint32_t b = p.edge_target[e0];
    const int64_t n_src = p.edge_count[e0];
    const uint32_t* src = p.sources + p.edge_start[e0];
    if (lane == 0) p.tgt_count[b] = 0;                   // left as the next batch expects it

    const uint32_t v = lane < p.R ? p.adj[(int64_t)b * p.R + lane] : EMPTY_ID;
    rowcopy[lane] = v;
    const uint64_t occupied = __ballot(v != EMPTY_ID);
    const int deg = __popcll(occupied);
    const uint32_t* cb = reinterpret_cast<const uint32_t*>(p.codes + (int64_t)b * ((ENC == ENC_SIGN1 ? 1 : 2) * NW_T));  // wave-uniform
    bsync();

    int cnt = 0;  // new candidates in buf[0..cnt)
    for (int64_t q = 0; q < n_src; q += 64) {
        const bool in_run = q + lane < n_src;
        const uint32_t t = in_run ? src[q + lane] : EMPTY_ID;
        bool ok = in_run && t != b;
        for (int j = 0; j < p.R; ++j) ok &= rowcopy[j] != t;
        const uint32_t dt = ok ? dist_uniform_vs_row<ENC, NW_T>(cb, p.codes, t) : 0u;
        const uint64_t om = __ballot(ok);
        const int m = __popcll(om);
        if (cnt + m > BUF) {  // make room: keep the nearest MAX_NEW seen so far
            for (int e = cnt + lane; e < BUF; e += 64) buf[e] = B_NONE;
            bsync();
            sort_keys(buf, BUF, lane);
            cnt = MAX_NEW;
        }
        if (ok) buf[cnt + __popcll(om & ((1ull << lane) - 1ull))] = ((uint64_t)dt << 32) | t;
        cnt += m;
        bsync();
    }
    if (cnt > MAX_NEW) {
        for (int e = cnt + lane; e < BUF; e += 64) buf[e] = B_NONE;
        bsync();
        sort_keys(buf, BUF, lane);
        cnt = MAX_NEW;
    }
    if (cnt == 0) return;
    if (deg + cnt <= p.R) {  // room for all: fill the free slots, nearest first (so that the row does not depend on
                             // the order in which the sources arrived); cnt <= 64, usually 1 to 3: rank by counting
        const uint64_t key = lane < cnt ? buf[lane] : B_NONE;
        int rank = 0;
        for (int j = 0; j < cnt; ++j) rank += buf[j] < key ? 1 : 0;
        if (lane < cnt) buf[64 + rank] = key;
        bsync();
        const bool free_slot = lane < p.R && v == EMPTY_ID;
        const int r = __popcll(__ballot(free_slot) & ((1ull << lane) - 1ull));
        if (free_slot && r < cnt) p.adj[(int64_t)b * p.R + lane] = (uint32_t)buf[64 + r];
        return;
    }
    // re-select from (old row U new candidates)
    const bool old = lane < p.R && v != EMPTY_ID;
    const uint32_t dv = old ? dist_uniform_vs_row<ENC, NW_T>(cb, p.codes, v) : 0u;
    if (old) buf[cnt + __popcll(occupied & ((1ull << lane) - 1ull))] = ((uint64_t)dv << 32) | v;
    const int total = cnt + deg;  // <= MAX_NEW + 64 = BUF
    const int m2 = pow2_at_least(total);
    for (int e = total + lane; e < m2; e += 64) buf[e] = B_NONE;
    bsync();
    sort_keys(buf, m2, lane);
    const int ns = select_edges_dev<ENC, NW_T>(p.codes, buf, total, p.R, p.alpha, sel, lane);
    if (lane < p.R) p.adj[(int64_t)b * p.R + lane] = lane < ns ? sel[lane] : EMPTY_ID;
}

// start of a construction: every adjacency slot empty, no edges counted at any target (a kernel, not memset nodes:
// the whole call may be captured into a graph)
__global__ void fill_empty_kernel(uint32_t* __restrict__ adj, int64_t words, uint32_t* __restrict__ tgt_count, int64_t n,
                                  uint32_t* __restrict__ cursor, uint32_t* __restrict__ bkt_count) {
    const int64_t at = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = at; i < words; i += step) adj[i] = EMPTY_ID;
    for (int64_t i = at; i < n; i += step) tgt_count[i] = 0;
    for (int64_t i = at; i < N_BUCKETS; i += step) bkt_count[i] = 0;
    if (at == 0) *cursor = 0;
}

// plane widths (64-bit words) the selection kernels are compiled for (a lane keeps a whole code in registers: 4 x width
// of them, which ends at 24 words); codes of other widths are zero-padded to the next one in the workspace
#define QV_BUILD_SM_WIDTHS(X) X(2) X(4) X(6) X(8) X(12) X(16) X(24)

int build_width_at_least(int nw, int encoding) {
    (void)encoding;   // every encoding is compiled for the same widths
    int best = 0;
#define QV_PICK(W) if (best == 0 && W >= nw) best = W;
    QV_BUILD_SM_WIDTHS(QV_PICK)
#undef QV_PICK
    return best;
}

template <int ENC, int NW_T>
static hipError_t launch_batch(const BuildParams& bp, hipStream_t stream) {
    hipLaunchKernelGGL((forward_select_kernel<ENC, NW_T>), dim3((unsigned)bp.bs), dim3(64), 0, stream, bp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t n_edges = bp.bs * bp.R;
    const dim3 per_edge((unsigned)((n_edges + 255) / 256));
    hipLaunchKernelGGL(reserve_segments_kernel, per_edge, dim3(256), 0, stream, bp, n_edges);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(bucket_offsets_kernel, dim3(1), dim3(N_BUCKETS), 0, stream, bp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(scatter_sources_kernel, per_edge, dim3(256), 0, stream, bp, n_edges);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL((reverse_kernel<ENC, NW_T>), dim3((unsigned)n_edges), dim3(64), 0, stream, bp);
    return hipGetLastError();
}

hipError_t launch_build_batch(int nw, int encoding, const BuildParams& bp, hipStream_t stream) {
#define QV_CASE_E(E, W) case W: return launch_batch<E, W>(bp, stream);
#define QV_CASE_S1(W) QV_CASE_E(ENC_SIGN1, W)
#define QV_CASE_SQ(W) QV_CASE_E(ENC_SQ2, W)
#define QV_CASE_SM(W) QV_CASE_E(ENC_SM, W)
    if (encoding == ENC_SIGN1) {
        switch (nw) { QV_BUILD_SM_WIDTHS(QV_CASE_S1) default: return hipErrorInvalidValue; }
    }
    if (encoding == ENC_SQ2) {
        switch (nw) { QV_BUILD_SM_WIDTHS(QV_CASE_SQ) default: return hipErrorInvalidValue; }
    }
    switch (nw) { QV_BUILD_SM_WIDTHS(QV_CASE_SM) default: return hipErrorInvalidValue; }
#undef QV_CASE_S1
#undef QV_CASE_SQ
#undef QV_CASE_SM
#undef QV_CASE_E
}

// ---- host loop -------------------------------------------------------------------------------

static size_t up256(size_t v) { return (v + 255) / 256 * 256; }

int64_t build_max_batch(int64_t n, int64_t max_batch) {
    int64_t b = n / 50;
    if (b < 1) b = 1;
    if (b > max_batch) b = max_batch;
    return b;
}

// bytes of the zero-padded copy of the codes (0 when the width is compiled for as it is)
static size_t padded_codes_bytes(int64_t n, int nw, int encoding) {
    const int pw = build_width_at_least(nw, encoding);
    return pw == nw ? 0 : up256((size_t)n * code_row_words(pw, encoding) * 8);
}

size_t build_workspace_bytes(int64_t n, int nw, int encoding, int R, int L, int64_t max_batch) {
    const int64_t mb = build_max_batch(n, max_batch);
    return up256((size_t)mb * L * 4) * 2 + up256((size_t)mb * 4) * 2 + up256((size_t)mb * R * 4) * 7 +
           up256((size_t)n * 4) * 2 + 256 + up256((size_t)(2 * N_BUCKETS + 1) * 4) + padded_codes_bytes(n, nw, encoding) + 256;
}

hipError_t build_graph(const uint64_t* codes, int64_t n, int d, int encoding, int R, int L, double alpha, uint32_t entry,
                       int64_t max_batch, uint32_t* adj, void* workspace, hipStream_t stream) {
    int nw = (d + 63) / 64;
    const int64_t mb = build_max_batch(n, max_batch);
    char* ws = static_cast<char*>(workspace);
    hipError_t e;
    if (const int pw = build_width_at_least(nw, encoding); pw != nw) {
        // planes padded with zero words to a width the selection kernels are compiled for: no distance changes
        if (pw == 0) return hipErrorInvalidValue;
        uint64_t* padded = reinterpret_cast<uint64_t*>(ws);
        ws += padded_codes_bytes(n, nw, encoding);
        e = launch_pad_codes(codes, n, nw, encoding == ENC_SIGN1 ? 1 : 2, pw, code_row_words(pw, encoding), padded, stream);
        if (e != hipSuccess) return e;
        codes = padded;
        nw = pw;
    }
    uint32_t* cand_ids = reinterpret_cast<uint32_t*>(ws);   ws += up256((size_t)mb * L * 4);
    uint32_t* cand_dist = reinterpret_cast<uint32_t*>(ws);  ws += up256((size_t)mb * L * 4);
    uint32_t* n_cand = reinterpret_cast<uint32_t*>(ws);     ws += up256((size_t)mb * 4);
    uint32_t* order = reinterpret_cast<uint32_t*>(ws);      ws += up256((size_t)mb * 4);
    uint32_t* edge_target = reinterpret_cast<uint32_t*>(ws);  ws += up256((size_t)mb * R * 4);
    uint32_t* edge_rank = reinterpret_cast<uint32_t*>(ws);    ws += up256((size_t)mb * R * 4);
    uint32_t* sources = reinterpret_cast<uint32_t*>(ws);      ws += up256((size_t)mb * R * 4);
    uint32_t* edge_start = reinterpret_cast<uint32_t*>(ws);   ws += up256((size_t)mb * R * 4);
    uint32_t* edge_count = reinterpret_cast<uint32_t*>(ws);   ws += up256((size_t)mb * R * 4);
    uint32_t* tgt_count = reinterpret_cast<uint32_t*>(ws);    ws += up256((size_t)n * 4);
    uint32_t* tgt_start = reinterpret_cast<uint32_t*>(ws);    ws += up256((size_t)n * 4);
    uint32_t* edge_bpos = reinterpret_cast<uint32_t*>(ws);    ws += up256((size_t)mb * R * 4);
    uint32_t* owner_list = reinterpret_cast<uint32_t*>(ws);   ws += up256((size_t)mb * R * 4);
    uint32_t* bkt_count = reinterpret_cast<uint32_t*>(ws);
    uint32_t* bkt_offset = bkt_count + N_BUCKETS;             ws += up256((size_t)(2 * N_BUCKETS + 1) * 4);
    uint32_t* cursor = reinterpret_cast<uint32_t*>(ws);

    {
        const int64_t words = n * (int64_t)R;
        const unsigned blocks = (unsigned)((words + 256 * 8 - 1) / (256 * 8) < 256 * 16 ? (words + 256 * 8 - 1) / (256 * 8) : 256 * 16);
        hipLaunchKernelGGL(fill_empty_kernel, dim3(blocks > 0 ? blocks : 1), dim3(256), 0, stream, adj, words, tgt_count, n, cursor, bkt_count);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    SearchParams sp{};
    sp.adj = adj; sp.codes = codes; sp.encoding = encoding; sp.row_stride = code_row_words(nw, encoding); sp.n = n; sp.nw = nw; sp.R = R; sp.entry = entry; sp.ef = L;
    sp.cand_ids = cand_ids; sp.cand_dist = cand_dist; sp.n_cand = n_cand;
    sp.n_expanded = nullptr; sp.n_evals = nullptr; sp.status = nullptr; sp.visit_order = nullptr; sp.visit_cap = 0;
    sp.order = nullptr;
    plan_visited_table(sp, 4096, true, true);  // visited set as a cache: same lists, more queries per compute unit
    BuildParams bp{};
    bp.codes = codes; bp.adj = adj; bp.n = n; bp.R = R; bp.L = L; bp.alpha = alpha;
    bp.cand_ids = cand_ids; bp.cand_dist = cand_dist; bp.n_cand = n_cand;
    bp.edge_target = edge_target; bp.edge_rank = edge_rank; bp.sources = sources; bp.tgt_count = tgt_count;
    bp.tgt_start = tgt_start; bp.cursor = cursor; bp.edge_start = edge_start; bp.edge_count = edge_count;
    bp.edge_bpos = edge_bpos; bp.owner_list = owner_list; bp.bkt_count = bkt_count; bp.bkt_offset = bkt_offset;
    bp.bkt_shift = 0;
    while (((int64_t)N_BUCKETS << bp.bkt_shift) < n) bp.bkt_shift++;
    for (int64_t done = 0; done < n;) {
        int64_t bs = done / 50;
        if (bs < 1) bs = 1;
        if (bs > mb) bs = mb;
        if (done + bs > n) bs = n - done;
        sp.qcodes = codes + done * (int64_t)code_row_words(nw, encoding);
        sp.nq = bs;
        sp.order = launch_query_order(sp, order, nullptr, nullptr, stream, &e) ? order : nullptr;   // long searches first (large batches only)
        if (e != hipSuccess) return e;
        e = launch_beam_search(sp, 0, stream);
        if (e != hipSuccess) return e;
        bp.done = done; bp.bs = bs;
        e = launch_build_batch(nw, encoding, bp, stream);
        if (e != hipSuccess) return e;
        done += bs;
    }
    return hipSuccess;
}

}  // namespace qv
