// Stage 2 of the query path (paper Sec. 3.3): exact cosine similarity between the float32 query and
// each member of the final candidate list, best k by (score descending, id ascending).
//
// One 256-thread workgroup per query; each of its four wavefronts takes every fourth candidate and
// streams that candidate's float32 row with fully coalesced loads (the row is contiguous, so this
// is a bandwidth-bound gather of ef rows of 4*d bytes).  Dot product and both squared norms are
// accumulated in double and the quotient is rounded to float once, so scores agree with a
// double-precision reference to the last float bit or so whatever the summation order.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "kernels.h"

namespace qv {

constexpr int RR_THREADS = 256;
constexpr int RR_WAVES = RR_THREADS / 64;
constexpr int RR_MAX_EF = 1024;

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__device__ __forceinline__ bool ranks_before(float sa, uint32_t ia, float sb, uint32_t ib) {
    return sa > sb || (sa == sb && ia < ib);
}

// (score, id) as one integer whose order is the ranking order: larger = earlier (score descending, then id
// ascending).  Floats map to integers of the same order (negative zero counts as zero, as in ranks_before);
// no key is 0, which stands for "no candidate".
__device__ __forceinline__ uint64_t rank_key(float s, uint32_t id) {
    uint32_t u = __float_as_uint(s + 0.0f);
    u ^= (u >> 31) ? 0xFFFFFFFFu : 0x80000000u;
    return ((uint64_t)u << 32) | (uint32_t)~id;
}
__device__ __forceinline__ float score_of_rank_key(uint64_t key) {
    uint32_t u = (uint32_t)(key >> 32);
    u ^= (u >> 31) ? 0x80000000u : 0xFFFFFFFFu;
    return __uint_as_float(u);
}

__global__ __launch_bounds__(RR_THREADS) void rerank_kernel(RerankParams p) {
    __shared__ float s_score[RR_MAX_EF];
    __shared__ uint32_t s_id[RR_MAX_EF];
    const int64_t q = blockIdx.x;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int d = p.d;
    const float* qv = p.queries + q * (int64_t)d;
    const int nc = (int)p.n_cand[q];
    const uint32_t* cand = p.cand_ids + q * (int64_t)p.ef;
    const bool vec4 = (d & 3) == 0;

    double qq = 0.0;
    if (vec4) {
        const float4* q4 = reinterpret_cast<const float4*>(qv);
        for (int i = lane; i < (d >> 2); i += 64) {
            float4 a = q4[i];
            qq += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
        }
    } else {
        for (int i = lane; i < d; i += 64) qq += (double)qv[i] * (double)qv[i];
    }
    qq = wave_sum_f64(qq);

    for (int c = wv; c < nc; c += RR_WAVES) {
        const uint32_t id = cand[c];
        const float* xv = p.vecs + (int64_t)id * d;
        double dot = 0.0, xx = 0.0;
        if (vec4) {
            const float4* x4 = reinterpret_cast<const float4*>(xv);
            const float4* q4 = reinterpret_cast<const float4*>(qv);
            for (int i = lane; i < (d >> 2); i += 64) {
                float4 a = x4[i], b = q4[i];
                dot += (double)a.x * b.x + (double)a.y * b.y + (double)a.z * b.z + (double)a.w * b.w;
                xx += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
            }
        } else {
            for (int i = lane; i < d; i += 64) {
                double a = xv[i];
                dot += a * (double)qv[i];
                xx += a * a;
            }
        }
        dot = wave_sum_f64(dot);
        xx = wave_sum_f64(xx);
        if (lane == 0) {
            float s = 0.0f;
            if (qq != 0.0 && xx != 0.0) s = (float)(dot / (sqrt(qq) * sqrt(xx)));
            if (s != s) s = -INFINITY;   // a stored vector with Inf or NaN in it ranks last (ties by id)
            s_score[c] = s;
            s_id[c] = id;
        }
    }
    __syncthreads();

    // The best k.  Few out of many (k <= candidates / 16, e.g. 10 of 1,024): k rounds of "take the best that is
    // left" -- every thread keeps its up to four candidates as sortable keys, a round is one maximum over the
    // workgroup -- instead of ranking every candidate against all others, which at 1,024 candidates costs a million
    // comparisons per query (a third of this kernel's time there).
    if (p.k * 16 <= nc) {
        __shared__ uint64_t s_best[2][RR_WAVES];
        uint64_t mine[RR_MAX_EF / RR_THREADS];
#pragma unroll
        for (int i = 0; i < RR_MAX_EF / RR_THREADS; ++i) {
            const int t = (int)threadIdx.x + i * RR_THREADS;
            mine[i] = t < nc ? rank_key(s_score[t], s_id[t]) : 0ull;
        }
        for (int r = 0; r < p.k; ++r) {   // k <= nc here
            uint64_t best = mine[0];
#pragma unroll
            for (int i = 1; i < RR_MAX_EF / RR_THREADS; ++i) best = mine[i] > best ? mine[i] : best;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const uint64_t other = __shfl_xor(best, off);
                best = other > best ? other : best;
            }
            if (lane == 0) s_best[r & 1][wv] = best;   // two buffers: one barrier per round is enough
            __syncthreads();
            best = s_best[r & 1][0];
#pragma unroll
            for (int w = 1; w < RR_WAVES; ++w) best = s_best[r & 1][w] > best ? s_best[r & 1][w] : best;
#pragma unroll
            for (int i = 0; i < RR_MAX_EF / RR_THREADS; ++i)
                if (mine[i] == best) mine[i] = 0ull;   // ids in a list are distinct, so keys are
            if (threadIdx.x == 0) {
                p.ids[q * (int64_t)p.k + r] = ~(uint32_t)best;
                p.scores[q * (int64_t)p.k + r] = score_of_rank_key(best);
            }
        }
        return;
    }

    // rank by counting: position of candidate t = number of candidates that come before it
    for (int t = threadIdx.x; t < nc; t += RR_THREADS) {
        float st = s_score[t];
        uint32_t it = s_id[t];
        int rank = 0;
        for (int j = 0; j < nc; ++j) rank += ranks_before(s_score[j], s_id[j], st, it) ? 1 : 0;
        if (rank < p.k) {
            p.ids[q * (int64_t)p.k + rank] = it;
            p.scores[q * (int64_t)p.k + rank] = st;
        }
    }
    for (int r = nc + threadIdx.x; r < p.k; r += RR_THREADS) {
        p.ids[q * (int64_t)p.k + r] = EMPTY_ID;
        p.scores[q * (int64_t)p.k + r] = -INFINITY;
    }
}

hipError_t launch_rerank(const RerankParams& p, hipStream_t stream) {
    if (p.nq == 0) return hipSuccess;
    if (p.ef > RR_MAX_EF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rerank_kernel, dim3((unsigned)p.nq), dim3(RR_THREADS), 0, stream, p);
    return hipGetLastError();
}

}  // namespace qv
