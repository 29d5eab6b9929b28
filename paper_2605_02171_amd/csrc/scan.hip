// Brute-force scan in code space (paper Sec. 6, "Practical compatibility test"; Sec. 5.5, Table 10
// "Top-10 overlap"): for every query code, the K base codes with the smallest (distance, id).
//
// All-pairs distances are arithmetic-bound, not bandwidth-bound: a base code is reused by every query.
// One lane owns one query (its code lives in registers), a wave owns 64 queries and walks a chunk of
// the base codes; the base code of the moment is the same for all lanes, so it is fetched with scalar
// loads and costs no vector memory traffic at all.  Each lane keeps its K best keys (dist << 32 | id)
// sorted in registers; a key below the lane's current worst is bubbled in.  A second small kernel
// merges the per-chunk lists of a query.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace qv {

constexpr uint64_t SCAN_NONE = ~0ull;

template <int KMAX>
__device__ __forceinline__ void bubble_in(uint64_t (&best)[KMAX], uint64_t key) {
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        const bool lt = key < best[j];
        const uint64_t lo = lt ? key : best[j];
        key = lt ? best[j] : key;
        best[j] = lo;
    }
}

// one 32-bit step of the distance under each encoding (see code_accumulate in the search kernel for the algebra):
// c0, c1: the base row's first / second plane dword; q0, q1, q2: the query's dwords (SQ2: (hi|lo), hi, (hi&lo))
template <int ENC>
__device__ __forceinline__ void scan_accumulate(uint32_t c0, uint32_t c1w, uint32_t q0, uint32_t q1, uint32_t q2,
                                                uint32_t& c1, uint32_t& c2, uint32_t& c3) {
    if constexpr (ENC == ENC_SM) {
        const uint32_t x = c0 ^ q0;
        c1 += __popc(x);
        c2 += __popc(__builtin_amdgcn_bitop3_b32(x, c1w, q1, 0xE0));   // x & (sv | sq)
        c3 += __popc(__builtin_amdgcn_bitop3_b32(x, c1w, q1, 0x80));   // x & sv & sq
    } else if constexpr (ENC == ENC_SIGN1) {
        c1 += __popc(c0 ^ q0);
    } else {
        c1 += __popc(__builtin_amdgcn_bitop3_b32(c1w, c0, q0, 0x56));  // (hi | lo) ^ q0
        c2 += __popc(c1w ^ q1);
        c3 += __popc(__builtin_amdgcn_bitop3_b32(c1w, c0, q2, 0x6A));  // (hi & lo) ^ q2
    }
}

// NW_T: 64-bit words per plane when known at compile time (query code in registers), 0: any (code in LDS)
template <int ENC, int NW_T, int KMAX>
__global__ __launch_bounds__(64) void bq_scan_kernel(const uint64_t* __restrict__ codes, int64_t n, int nw,
                                                     const uint64_t* __restrict__ qcodes, int64_t nq, int K,
                                                     int64_t chunk, uint64_t* __restrict__ partial) {
    extern __shared__ uint32_t qlds[];  // generic path: [6*nw][64] dwords, word-major
    const int lane = threadIdx.x;
    const int64_t qi = (int64_t)blockIdx.x * 64 + lane;
    const bool live = qi < nq;
    const int NW = NW_T > 0 ? NW_T : nw;
    const int DW = 2 * NW;  // dwords per plane
    constexpr int DW_T = NW_T > 0 ? 2 * NW_T : 1;
    constexpr int PLANES = ENC == ENC_SIGN1 ? 1 : 2;
    uint32_t qp[DW_T], qs[DW_T], q3[DW_T];
    const uint32_t* qsrc = reinterpret_cast<const uint32_t*>(qcodes + (live ? qi : 0) * (int64_t)(PLANES * NW));
    auto prepare = [&](int w, uint32_t& q0, uint32_t& q1, uint32_t& q2) {
        const uint32_t a = qsrc[w], b = PLANES == 2 ? qsrc[DW + w] : 0u;
        if constexpr (ENC == ENC_SQ2) { q0 = a | b; q1 = b; q2 = a & b; }
        else { q0 = a; q1 = b; q2 = 0u; }
    };
    if constexpr (NW_T > 0) {
#pragma unroll
        for (int w = 0; w < DW_T; ++w) prepare(w, qp[w], qs[w], q3[w]);
    } else {
        for (int w = 0; w < DW; ++w) {
            uint32_t q0, q1, q2;
            prepare(w, q0, q1, q2);
            qlds[w * 64 + lane] = q0; qlds[(DW + w) * 64 + lane] = q1; qlds[(2 * DW + w) * 64 + lane] = q2;
        }
        qp[0] = qs[0] = q3[0] = 0;
    }
    uint64_t best[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) best[j] = SCAN_NONE;
    uint64_t worst = SCAN_NONE;  // best[K-1]

    const int64_t lo = (int64_t)blockIdx.y * chunk;
    const int64_t hi = lo + chunk < n ? lo + chunk : n;
    for (int64_t row = lo; row < hi; ++row) {
        const uint32_t* c = reinterpret_cast<const uint32_t*>(codes + row * (int64_t)(PLANES * NW));  // wave-uniform
        uint32_t c1 = 0, c2 = 0, c3 = 0;
        if constexpr (NW_T > 0) {
#pragma unroll
            for (int w = 0; w < DW_T; ++w)
                scan_accumulate<ENC>(c[w], PLANES == 2 ? c[DW_T + w] : 0u, qp[w], qs[w], q3[w], c1, c2, c3);
        } else {
            for (int w = 0; w < DW; ++w)
                scan_accumulate<ENC>(c[w], PLANES == 2 ? c[DW + w] : 0u, qlds[w * 64 + lane], qlds[(DW + w) * 64 + lane],
                                     qlds[(2 * DW + w) * 64 + lane], c1, c2, c3);
        }
        const uint64_t key = ((uint64_t)(ENC == ENC_SM ? c1 + c2 + 2u * c3 : c1 + c2 + c3) << 32) | (uint32_t)row;
        if (key < worst) {
            bubble_in<KMAX>(best, key);
#pragma unroll
            for (int j = 0; j < KMAX; ++j)
                if (j == K - 1) worst = best[j];
        }
    }
    if (live) {
        uint64_t* out = partial + ((int64_t)blockIdx.y * nq + qi) * K;
#pragma unroll
        for (int j = 0; j < KMAX; ++j)
            if (j < K) out[j] = best[j];
    }
}

// one wave per query: the K smallest of its nchunks * K partial keys, by repeated minimum
__global__ __launch_bounds__(64) void bq_scan_merge_kernel(const uint64_t* __restrict__ partial, int64_t nq, int K,
                                                           int nchunks, uint32_t* __restrict__ ids,
                                                           uint32_t* __restrict__ dist) {
    const int lane = threadIdx.x;
    const int64_t q = blockIdx.x;
    const int total = nchunks * K;
    uint64_t last = 0;
    bool first = true;
    for (int r = 0; r < K; ++r) {
        uint64_t m = SCAN_NONE;
        for (int i = lane; i < total; i += 64) {
            const int ch = i / K, j = i - ch * K;
            const uint64_t key = partial[((int64_t)ch * nq + q) * K + j];
            if ((first || key > last) && key < m) m = key;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint32_t l = (uint32_t)__shfl_xor((int)(uint32_t)m, off);
            const uint32_t h = (uint32_t)__shfl_xor((int)(uint32_t)(m >> 32), off);
            const uint64_t o = ((uint64_t)h << 32) | l;
            m = o < m ? o : m;
        }
        if (lane == 0) {
            ids[q * K + r] = m == SCAN_NONE ? EMPTY_ID : (uint32_t)m;
            dist[q * K + r] = m == SCAN_NONE ? EMPTY_ID : (uint32_t)(m >> 32);
        }
        if (m == SCAN_NONE) {  // nothing left: pad the rest
            if (lane == 0)
                for (int t = r + 1; t < K; ++t) { ids[q * K + t] = EMPTY_ID; dist[q * K + t] = EMPTY_ID; }
            break;
        }
        last = m;
        first = false;
    }
}

// out[q] = number of entries of a[q][0..K) that also occur in b[q][0..K) (EMPTY never matches)
__global__ void topk_overlap_kernel(const uint32_t* __restrict__ a, const uint32_t* __restrict__ b, int64_t nq, int K,
                                    uint32_t* __restrict__ out) {
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nq) return;
    uint32_t hits = 0;
    for (int i = 0; i < K; ++i) {
        const uint32_t x = a[q * K + i];
        if (x == EMPTY_ID) continue;
        for (int j = 0; j < K; ++j)
            if (b[q * K + j] == x) { hits++; break; }
    }
    out[q] = hits;
}

int64_t bq_scan_chunk_rows(int64_t n) {
    // enough chunks to fill the chip even with few queries, never fewer than 1024 rows per chunk
    int64_t chunk = (n + 63) / 64;
    if (chunk < 1024) chunk = 1024;
    if (chunk > 16384) chunk = 16384;
    return chunk;
}

template <int ENC, int NW_T>
static hipError_t launch_scan_k(const uint64_t* codes, int64_t n, int nw, const uint64_t* qcodes, int64_t nq, int K,
                                int64_t chunk, uint64_t* partial, hipStream_t stream) {
    dim3 grid((unsigned)((nq + 63) / 64), (unsigned)((n + chunk - 1) / chunk));
    size_t lds = NW_T > 0 ? 0 : (size_t)nw * 6 * 64 * 4;
    if (K <= 16) {
        auto kern = bq_scan_kernel<ENC, NW_T, 16>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, grid, dim3(64), lds, stream, codes, n, nw, qcodes, nq, K, chunk, partial);
    } else {
        auto kern = bq_scan_kernel<ENC, NW_T, 64>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, grid, dim3(64), lds, stream, codes, n, nw, qcodes, nq, K, chunk, partial);
    }
    return hipGetLastError();
}

hipError_t launch_bq_scan(const uint64_t* codes, int64_t n, int d, int encoding, const uint64_t* qcodes, int64_t nq, int K,
                          uint64_t* partial, uint32_t* ids, uint32_t* dist, hipStream_t stream) {
    if (nq == 0) return hipSuccess;
    const int nw = (d + 63) / 64;
    const int64_t chunk = bq_scan_chunk_rows(n);
    const int nchunks = n > 0 ? (int)((n + chunk - 1) / chunk) : 0;
    hipError_t e = hipSuccess;
    if (n > 0) {
#define QV_SCAN_WIDTHS(E) \
        switch (nw) { \
            case 2: e = launch_scan_k<E, 2>(codes, n, nw, qcodes, nq, K, chunk, partial, stream); break; \
            case 6: e = launch_scan_k<E, 6>(codes, n, nw, qcodes, nq, K, chunk, partial, stream); break; \
            case 8: e = launch_scan_k<E, 8>(codes, n, nw, qcodes, nq, K, chunk, partial, stream); break; \
            case 12: e = launch_scan_k<E, 12>(codes, n, nw, qcodes, nq, K, chunk, partial, stream); break; \
            case 16: e = launch_scan_k<E, 16>(codes, n, nw, qcodes, nq, K, chunk, partial, stream); break; \
            default: e = launch_scan_k<E, 0>(codes, n, nw, qcodes, nq, K, chunk, partial, stream); break; \
        }
        if (encoding == ENC_SIGN1) { QV_SCAN_WIDTHS(ENC_SIGN1) }
        else if (encoding == ENC_SQ2) { QV_SCAN_WIDTHS(ENC_SQ2) }
        else { QV_SCAN_WIDTHS(ENC_SM) }
#undef QV_SCAN_WIDTHS
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(bq_scan_merge_kernel, dim3((unsigned)nq), dim3(64), 0, stream, partial, nq, K, nchunks, ids, dist);
    return hipGetLastError();
}

hipError_t launch_topk_overlap(const uint32_t* a, const uint32_t* b, int64_t nq, int K, uint32_t* out,
                               hipStream_t stream) {
    if (nq == 0) return hipSuccess;
    hipLaunchKernelGGL(topk_overlap_kernel, dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, stream, a, b, nq, K, out);
    return hipGetLastError();
}

}  // namespace qv
