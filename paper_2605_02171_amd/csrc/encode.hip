// 2-bit Sign-Magnitude encoder (paper Sec. 3.1, the two encoding equations) for gfx950.
//
// One wavefront encodes one vector.  Lane l of the wave owns dimensions l, l+64, l+128, ...,
// so every load instruction reads 256 contiguous bytes and a wave-wide ballot of a
// per-dimension predicate *is* the 64-bit word of the bit-plane (bit l = dimension 64w+l).
//
// The threshold test uses the exact mean: strong_i <=> d*|x_i| > sum_j |x_j| in real
// arithmetic.  Fast path: the sum is accumulated in double (every term is >= 0, so any
// summation order has relative error <= (d-1)*2^-53) and d*|x_i| is exact in double; a
// comparison whose gap exceeds d*2^-52*sum is therefore certain.  Any vector with a
// comparison inside that band is redone with an integer super-accumulator in LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace qv {

constexpr int ENC_WAVES = 4;     // waves (vectors) per workgroup
constexpr int EXACT_LIMBS = 12;  // 32-bit digits of the exact sum, in units of 2^-149

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// |x| = m * 2^(sh-149), m < 2^24; returns false for Inf/NaN
__device__ __forceinline__ bool split_abs(float x, uint32_t& m, int& sh) {
    uint32_t u = __float_as_uint(x);
    uint32_t e = (u >> 23) & 0xFFu, f = u & 0x7FFFFFu;
    if (e == 0xFFu) { m = 0; sh = 0; return false; }
    if (e == 0) { m = f; sh = 0; } else { m = f | 0x800000u; sh = (int)e - 1; }
    return true;
}

// |x| as a double, built from the integer fields so that float32 subnormals never depend on the
// float denormal mode (0 for Inf/NaN)
__device__ __forceinline__ double abs_as_double(float x) {
    uint32_t m; int sh;
    split_abs(x, m, sh);
    return ldexp((double)m, sh - 149);
}

__device__ __forceinline__ bool is_positive(float x) { return (int32_t)__float_as_uint(x) > 0; }

__global__ __launch_bounds__(64 * ENC_WAVES) void encode_kernel(const float* __restrict__ x, int64_t n, int d,
                                                                uint64_t* __restrict__ codes,
                                                                uint32_t* __restrict__ status) {
    __shared__ unsigned long long acc[ENC_WAVES][EXACT_LIMBS];
    __shared__ uint32_t digits[ENC_WAVES][EXACT_LIMBS];
    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    const int64_t v = (int64_t)blockIdx.x * ENC_WAVES + wv;
    if (v >= n) return;  // whole wave leaves together; no block-wide barrier is used below
    const int W = (d + 63) >> 6;
    const float* xv = x + v * (int64_t)d;
    uint64_t* cv = codes + v * (int64_t)(2 * W);

    // pass 1: sum of magnitudes in double
    double part = 0.0;
    bool finite = true;
    for (int i = lane; i < d; i += 64) {
        float xi = xv[i];
        finite &= (__float_as_uint(xi) & 0x7F800000u) != 0x7F800000u;
        part += abs_as_double(xi);
    }
    const double S = wave_sum(part);
    const bool all_finite = __all(finite);
    const double margin = (double)d * 0x1p-52 * S;

    // pass 2 (the row is in L1/L2 now): bit-planes by ballot
    bool doubtful = false;
    for (int w = 0; w < W; ++w) {
        int i = (w << 6) + lane;
        float xi = i < d ? xv[i] : 0.0f;
        double t = (double)d * abs_as_double(xi);
        bool strong = t > S;
        doubtful |= (i < d) && (fabs(t - S) <= margin);
        uint64_t pw = __ballot(is_positive(xi));
        uint64_t sw = __ballot(strong);
        if (lane == 0) cv[w] = pw;
        if (lane == 1) cv[W + w] = sw;
    }
    if (status && lane == 0) status[v] = all_finite ? 0u : QV_STATUS_NONFINITE_BIT;
    if (!all_finite || !__any(doubtful)) return;

    // exact redo of the magnitude plane: S as an integer in units of 2^-149
    if (lane < EXACT_LIMBS) acc[wv][lane] = 0ull;
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < d; i += 64) {
        uint32_t m; int sh;
        split_abs(xv[i], m, sh);
        unsigned long long val = (unsigned long long)m << (sh & 31);  // < 2^55
        atomicAdd(&acc[wv][sh >> 5], val & 0xFFFFFFFFull);
        atomicAdd(&acc[wv][(sh >> 5) + 1], val >> 32);
    }
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) {
        unsigned long long carry = 0;
        for (int k = 0; k < EXACT_LIMBS; ++k) {
            unsigned long long s = acc[wv][k] + carry;  // each limb holds < d * 2^32 <= 2^49
            digits[wv][k] = (uint32_t)s;
            carry = s >> 32;
        }
    }
    __builtin_amdgcn_wave_barrier();
    for (int w = 0; w < W; ++w) {
        int i = (w << 6) + lane;
        float xi = i < d ? xv[i] : 0.0f;
        uint32_t m; int sh;
        split_abs(xi, m, sh);
        // T = d * m * 2^sh occupies digits k0, k0+1, k0+2
        unsigned long long dm = (unsigned long long)m * (unsigned long long)d;  // < 2^41
        int k0 = sh >> 5, b = sh & 31;
        uint32_t t0 = (uint32_t)(dm << b);
        uint32_t t1 = (uint32_t)((dm << b) >> 32);
        uint32_t t2 = b ? (uint32_t)(dm >> (64 - b)) : 0u;
        int cmp = 0;  // sign of T - S
        for (int k = EXACT_LIMBS - 1; k >= 0 && cmp == 0; --k) {
            uint32_t tk = k == k0 ? t0 : (k == k0 + 1 ? t1 : (k == k0 + 2 ? t2 : 0u));
            uint32_t sk = digits[wv][k];
            cmp = tk > sk ? 1 : (tk < sk ? -1 : 0);
        }
        uint64_t sw = __ballot(i < d && cmp > 0);
        if (lane == 1) cv[W + w] = sw;
    }
}

// out[p] = symmetric distance of code rows ia[p] (in a) and ib[p] (in b): one thread per pair
__global__ void bq_distance_kernel(const uint64_t* __restrict__ a, const int64_t* __restrict__ ia,
                                   const uint64_t* __restrict__ b, const int64_t* __restrict__ ib, int64_t npairs,
                                   int W, uint32_t* __restrict__ out) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= npairs) return;
    const uint64_t* ca = a + ia[p] * (int64_t)(2 * W);
    const uint64_t* cb = b + ib[p] * (int64_t)(2 * W);
    uint32_t c1 = 0, c2 = 0, c3 = 0;
    for (int w = 0; w < W; ++w) {
        uint64_t X = ca[w] ^ cb[w];
        uint64_t sa = ca[W + w], sb = cb[W + w];
        c1 += __popcll(X);
        c2 += __popcll(X & (sa | sb));
        c3 += __popcll(X & sa & sb);
    }
    out[p] = c1 + c2 + 2u * c3;
}

hipError_t launch_encode(const float* x, int64_t n, int d, uint64_t* codes, uint32_t* status, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    dim3 grid((unsigned)((n + ENC_WAVES - 1) / ENC_WAVES));
    hipLaunchKernelGGL(encode_kernel, grid, dim3(64 * ENC_WAVES), 0, stream, x, n, d, codes, status);
    return hipGetLastError();
}

hipError_t launch_bq_distance(const uint64_t* a, const int64_t* ia, const uint64_t* b, const int64_t* ib,
                              int64_t npairs, int d, uint32_t* out, hipStream_t stream) {
    if (npairs == 0) return hipSuccess;
    int W = (d + 63) / 64;
    dim3 grid((unsigned)((npairs + 255) / 256));
    hipLaunchKernelGGL(bq_distance_kernel, grid, dim3(256), 0, stream, a, ia, b, ib, npairs, W, out);
    return hipGetLastError();
}

}  // namespace qv
