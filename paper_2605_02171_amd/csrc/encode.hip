// 2-bit Sign-Magnitude encoder (paper Sec. 3.1, the two encoding equations) for gfx950.
//
// One wavefront encodes one vector (a few consecutive ones when they are short).  Lane l of the wave
// owns dimensions l, l+64, l+128, ..., so every load instruction reads 256 contiguous bytes and a
// wave-wide ballot of a per-dimension predicate *is* the 64-bit word of the bit-plane (bit l = dimension 64w+l).
//
// The threshold test uses the exact mean: strong_i <=> d*|x_i| > sum_j |x_j| in real
// arithmetic.  Fast path: the sum S is accumulated in double (every term is >= 0, so any
// summation order has relative error <= (d-1)*2^-53); with margin = d*2^-52*S, a value above
// (S+margin)/d is certainly strong and one below (S-margin)/d certainly weak.  Both bounds are
// rounded outwards to float32 (two ulps further than round-to-nearest, which also covers the 2^-52 of
// forming the quotients with a precomputed 1/d), so each element costs two float compares.  Any vector with an element between the bounds is redone with an integer
// super-accumulator in LDS.  (float32 subnormals are compared and converted as such: HIP's
// default for gfx9 keeps them; the parity tests cover subnormal-only vectors.)
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

// v_writelane_b32: `value` (wave-uniform) replaces lane `lane` of `old`; reached through the compiler's intrinsic so
// that the compiler keeps the wait states between the compare that produced `value` and this instruction
extern "C" __device__ int qv_writelane(int value, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

__device__ __forceinline__ bool is_positive(float x) { return (int32_t)__float_as_uint(x) > 0; }

// float32 bounds around S/d: |x| > hi => D*|x| > S + margin;  |x| < lo => D*|x| < S - margin
__device__ __forceinline__ void certain_bounds(double S, int d, float& lo, float& hi) {
    const double margin = (double)d * 0x1p-52 * S;
    const float h = (float)((S + margin) / (double)d);
    const float l = (float)((S - margin) / (double)d);
    hi = __uint_as_float(__float_as_uint(h) + 2u);   // Inf + 2 is a NaN: then nothing is "certainly strong"
    const uint32_t lb = __float_as_uint(l);
    lo = __uint_as_float(lb >= 2u ? lb - 2u : 0u);
}

// Exact redo of the magnitude plane of one vector (whole wave): S as an integer in units of 2^-149.
__device__ __forceinline__ void exact_magnitude_plane(const float* __restrict__ xv, int d, int W,
                                                      uint64_t* __restrict__ cv, unsigned long long* acc,
                                                      uint32_t* digits, int lane) {
    if (lane < EXACT_LIMBS) acc[lane] = 0ull;
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < d; i += 64) {
        uint32_t m; int sh;
        split_abs(xv[i], m, sh);
        unsigned long long val = (unsigned long long)m << (sh & 31);  // < 2^55
        atomicAdd(&acc[sh >> 5], val & 0xFFFFFFFFull);
        atomicAdd(&acc[(sh >> 5) + 1], val >> 32);
    }
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) {
        unsigned long long carry = 0;
        for (int k = 0; k < EXACT_LIMBS; ++k) {
            unsigned long long s = acc[k] + carry;  // each limb holds < d * 2^33 <= 2^49
            digits[k] = (uint32_t)s;
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
            uint32_t sk = digits[k];
            cmp = tk > sk ? 1 : (tk < sk ? -1 : 0);
        }
        uint64_t sw = __ballot(i < d && cmp > 0);
        if (lane == 1) cv[W + w] = sw;
    }
}

// Vectors of up to 64*W dimensions, W known at compile time: the whole vector sits in registers
// (W values per lane), all loads are issued before the first use, the row is read exactly once and
// the code words leave through one coalesced store.  The body has no branch but the rare exact redo:
// the ragged tail of the last word is clamped to the row's last element and zeroed, every
// per-dimension predicate is one compare whose wave-wide result (a scalar register pair) is the
// plane's word, the "in doubt" test is scalar arithmetic on those words, and the words are dropped into
// the lanes that store them.  A wave takes ROWS consecutive vectors (short rows: their independent
// reductions overlap and their 2W ROWS <= 64 code words, contiguous in memory, still leave in one store).
template <int W, int ROWS>
__global__ __launch_bounds__(64 * ENC_WAVES) void encode_kernel_reg(const float* __restrict__ x, int64_t n, int d,
                                                                    uint64_t* __restrict__ codes,
                                                                    uint32_t* __restrict__ status) {
    static_assert(ROWS == 1 || 2 * W * ROWS <= 64, "the code words of a wave's vectors must fit one register");
    __shared__ unsigned long long acc[ENC_WAVES][EXACT_LIMBS];
    __shared__ uint32_t digits[ENC_WAVES][EXACT_LIMBS];
    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    const int tail_i = (W - 1) * 64 + lane;                   // this lane's dimension in the last word
    const bool tail_valid = tail_i < d;
    const int tail_off = tail_valid ? tail_i : d - 1;
    const uint64_t tail_mask = __ballot(tail_valid);
    // 1/d rounded to nearest: (S +- margin) * inv_d is within 2^-52 of the quotient, far inside the two
    // float32 ulps by which the bounds are moved outwards
    const double inv_d = 1.0 / (double)d;
    const double margin_factor = (double)d * 0x1p-52;
    // No loop over vectors: with a body this short, many short-lived waves stream better than fewer waves
    // that prefetch their next row (1M x 768: 0.53 against 0.58 ms).
    const int64_t v0 = ((int64_t)blockIdx.x * ENC_WAVES + wv) * ROWS;
    if (v0 >= n) return;  // whole wave leaves together; no block-wide barrier is used below
    const int rows = n - v0 < ROWS ? (int)(n - v0) : ROWS;

    float xr[ROWS][W];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const float* xv = x + (v0 + (r < rows ? r : rows - 1)) * (int64_t)d;   // beyond the end: the last row again
#pragma unroll
        for (int w = 0; w < W - 1; ++w) xr[r][w] = __builtin_nontemporal_load(xv + (w << 6) + lane);
        xr[r][W - 1] = __builtin_nontemporal_load(xv + tail_off);
    }

    int w0_lo = 0, w0_hi = 0, w1_lo = 0, w1_hi = 0;   // lane l keeps code word l of the wave's vectors (and word 64 + l when 2W > 64)
    uint32_t redo = 0, nonfinite = 0;                  // bit r: vector r needs the exact redo / holds Inf or NaN
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        xr[r][W - 1] = tail_valid ? xr[r][W - 1] : 0.0f;
        double part = 0.0;
#pragma unroll
        for (int w = 0; w < W; ++w) part += (double)fabsf(xr[r][w]);
        const double S = wave_sum(part);                       // the same bits in every lane
        // finite magnitudes cannot overflow a double sum (d * 2^128 < 2^1024), so S tells whether all are
        const bool all_finite = S < __builtin_huge_val();
        const double margin = margin_factor * S;
        const float h = (float)((S + margin) * inv_d), l = (float)((S - margin) * inv_d);
        const float hi = __uint_as_float(__float_as_uint(h) + 2u);   // Inf + 2 is a NaN: then nothing is "certainly strong"
        const uint32_t lb = __float_as_uint(l);
        const float lo = __uint_as_float(lb >= 2u ? lb - 2u : 0u);

        uint64_t doubt = 0;                                    // scalar: dimensions neither certainly strong nor certainly weak
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const float a = fabsf(xr[r][w]);
            const uint64_t sw = __ballot(a > hi);
            const uint64_t ge = __ballot(a >= lo);
            const uint64_t pw = __ballot(is_positive(xr[r][w]));
            doubt |= (w == W - 1 ? ge & tail_mask : ge) & ~sw;
            const int at = r * 2 * W + w;
            w0_lo = qv_writelane((int)(uint32_t)pw, at, w0_lo);
            w0_hi = qv_writelane((int)(uint32_t)(pw >> 32), at, w0_hi);
            if (at + W < 64) {
                w0_lo = qv_writelane((int)(uint32_t)sw, at + W, w0_lo);
                w0_hi = qv_writelane((int)(uint32_t)(sw >> 32), at + W, w0_hi);
            } else {
                w1_lo = qv_writelane((int)(uint32_t)sw, at + W - 64, w1_lo);
                w1_hi = qv_writelane((int)(uint32_t)(sw >> 32), at + W - 64, w1_hi);
            }
        }
        if (!all_finite) nonfinite |= 1u << r;
        else if (doubt != 0) redo |= 1u << r;
    }
    uint64_t* cv = codes + v0 * (int64_t)(2 * W);
    if (lane < 2 * W * rows && lane < 64) cv[lane] = ((uint64_t)(uint32_t)w0_hi << 32) | (uint32_t)w0_lo;
    if (2 * W > 64 && lane < 2 * W - 64) cv[64 + lane] = ((uint64_t)(uint32_t)w1_hi << 32) | (uint32_t)w1_lo;
    if (status && lane < rows) status[v0 + lane] = (nonfinite >> lane) & 1u ? QV_STATUS_NONFINITE_BIT : 0u;
    if (redo != 0) {
        for (int r = 0; r < rows; ++r)
            if ((redo >> r) & 1u)
                exact_magnitude_plane(x + (v0 + r) * (int64_t)d, d, W, cv + r * 2 * W, acc[wv], digits[wv], lane);
    }
}

// Any dimension: two passes over the row (the second one hits cache), four loads in flight.
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
    for (int i0 = lane; i0 < d; i0 += 256) {
        float xi[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) xi[u] = i0 + 64 * u < d ? xv[i0 + 64 * u] : 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            finite &= (__float_as_uint(xi[u]) & 0x7F800000u) != 0x7F800000u;
            part += (double)fabsf(xi[u]);
        }
    }
    const double S = wave_sum(part);
    const bool all_finite = __all(finite);
    float lo, hi;
    certain_bounds(S, d, lo, hi);

    // pass 2 (the row is in L1/L2 now): bit-planes by ballot
    bool doubtful = false;
    for (int w = 0; w < W; ++w) {
        int i = (w << 6) + lane;
        float xi = i < d ? xv[i] : 0.0f;
        const float a = fabsf(xi);
        bool strong = a > hi;
        doubtful |= (i < d) && !strong && !(a < lo);
        uint64_t pw = __ballot(is_positive(xi));
        uint64_t sw = __ballot(strong);
        if (lane == 0) cv[w] = pw;
        if (lane == 1) cv[W + w] = sw;
    }
    if (status && lane == 0) status[v] = all_finite ? 0u : QV_STATUS_NONFINITE_BIT;
    if (!all_finite || !__any(doubtful)) return;
    exact_magnitude_plane(xv, d, W, cv, acc[wv], digits[wv], lane);
}

// ---- the two encodings of the paper's ablation (Sec. 5.5 "Encoding Ablation", Table 10) ----------------
// 1-bit sign: the sign plane alone.  One wave per vector, 64 dimensions per ballot.
__global__ __launch_bounds__(64 * ENC_WAVES) void encode_sign1_kernel(const float* __restrict__ x, int64_t n, int d,
                                                                      uint64_t* __restrict__ codes,
                                                                      uint32_t* __restrict__ status) {
    const int lane = threadIdx.x & 63;
    const int64_t v = (int64_t)blockIdx.x * ENC_WAVES + (threadIdx.x >> 6);
    if (v >= n) return;
    const int W = (d + 63) >> 6;
    const float* xv = x + v * (int64_t)d;
    bool finite = true;
    for (int w = 0; w < W; ++w) {
        const int i = (w << 6) + lane;
        const float xi = i < d ? xv[i] : 0.0f;
        finite &= (__float_as_uint(xi) & 0x7F800000u) != 0x7F800000u;
        const uint64_t pw = __ballot(is_positive(xi));
        if (lane == 0) codes[v * (int64_t)W + w] = pw;
    }
    const bool all_finite = __all(finite);
    if (status && lane == 0) status[v] = all_finite ? 0u : QV_STATUS_NONFINITE_BIT;
}

// 2-bit uniform quantiser of the paper's ablation (Sec. 5.5, Table 10; the paper names "four equal-width buckets" but no
// range).  Reading taken: the range is [-2 tau, +2 tau] with tau the vector's exact mean magnitude, so the bucket
// edges are -tau, 0, +tau; level 3 iff x > tau, 2 iff 0 < x <= tau, 1 iff -tau <= x <= 0, 0 iff x < -tau (the strict
// tests of Sec. 3.1).  These are the two decisions of the Sign-Magnitude code, so the levels follow from its planes
// (p = positive, s = strong): high bit = p, low bit = not (p xor s).  The kernel rewrites a Sign-Magnitude code row in
// place: planes become low bit, then high bit; bits of dimensions >= d stay 0.  One thread per plane word.
__global__ __launch_bounds__(256) void sq2_from_sm_kernel(uint64_t* __restrict__ codes, int64_t n, int d) {
    const int W = (d + 63) >> 6;
    const int64_t total = n * W;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / W;
        const int w = (int)(i - row * W);
        uint64_t* r = codes + row * (2 * W);
        const uint64_t p = r[w], s = r[W + w];
        const int live = d - (w << 6);   // dimensions this word holds
        const uint64_t mask = live >= 64 ? ~0ull : ((1ull << live) - 1ull);
        r[w] = ~(p ^ s) & mask;
        r[W + w] = p;
    }
}

// out[p] = distance of code rows ia[p] (in a) and ib[p] (in b) under the given encoding: one thread per pair
__global__ void bq_distance_kernel(const uint64_t* __restrict__ a, const int64_t* __restrict__ ia,
                                   const uint64_t* __restrict__ b, const int64_t* __restrict__ ib, int64_t npairs,
                                   int W, int encoding, uint32_t* __restrict__ out) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= npairs) return;
    const int rw = code_row_words_dev(W, encoding);
    const uint64_t* ca = a + ia[p] * (int64_t)rw;
    const uint64_t* cb = b + ib[p] * (int64_t)rw;
    uint32_t c1 = 0, c2 = 0, c3 = 0;
    for (int w = 0; w < W; ++w) {
        if (encoding == ENC_SIGN1) {
            c1 += __popcll(ca[w] ^ cb[w]);
        } else if (encoding == ENC_SQ2) {
            const uint64_t la = ca[w], ha = ca[W + w], lb = cb[w], hb = cb[W + w];
            c1 += __popcll((la | ha) ^ (lb | hb)) + __popcll((la & ha) ^ (lb & hb));
            c2 += __popcll(ha ^ hb);
        } else {
            uint64_t X = ca[w] ^ cb[w];
            uint64_t sa = ca[W + w], sb = cb[W + w];
            c1 += __popcll(X);
            c2 += __popcll(X & (sa | sb));
            c3 += __popcll(X & sa & sb);
        }
    }
    out[p] = c1 + c2 + 2u * c3;
}

// Measurement aid: every wave reads 64 rows of 2*NW words per round, rows named by ids[], with the access pattern
// of the search kernel's code gather for that width -- G lanes per row, lane s of a group taking a contiguous
// share of each plane in 16-byte loads when the shares are an even number of words (768-d: two lanes per row, three
// 16-byte loads per plane and lane), words s, s+G, ... in 8-byte loads otherwise; as many of the G passes in flight
// as the search kernel keeps -- and no arithmetic beyond an XOR fold, so its rate is what the memory system gives
// to that pattern.  NW = 0: any width, 4 lanes per row, 8-byte loads.
template <int NW, int G>
__global__ __launch_bounds__(64) void gather_probe_kernel(const uint64_t* __restrict__ codes, int row_words,
                                                          const uint32_t* __restrict__ ids, int64_t n_ids,
                                                          uint64_t* __restrict__ sink) {
    const int lane = threadIdx.x;
    uint64_t acc = 0;
    if constexpr (NW > 0) {
        constexpr int RPP = 64 / G, KW = (NW + G - 1) / G;
        constexpr int BATCH = (2 * KW * G <= 48) ? G : (48 / (2 * KW) > 0 ? 48 / (2 * KW) : 1);
        constexpr bool BLOCKED = BATCH == G && G <= 4 && NW % (2 * G) == 0;
        const int sub = lane % G, grp = lane / G;
        for (int64_t base = (int64_t)blockIdx.x * 64; base + 64 <= n_ids; base += (int64_t)gridDim.x * 64) {
            const uint32_t mine = ids[base + lane];
            for (int b0 = 0; b0 < G; b0 += BATCH) {
                uint64_t pv[BATCH][KW], sv[BATCH][KW];
#pragma unroll
                for (int b = 0; b < BATCH; ++b) {
                    if (b0 + b >= G) {   // wave-uniform: the last batch may be partial
#pragma unroll
                        for (int i = 0; i < KW; ++i) pv[b][i] = sv[b][i] = 0ull;
                        continue;
                    }
                    const uint32_t r = (uint32_t)__shfl((int)mine, (b0 + b) * RPP + grp);
                    const uint64_t* row = codes + (int64_t)r * (2 * NW);
                    if constexpr (BLOCKED) {
                        const uint4* r4 = reinterpret_cast<const uint4*>(row + sub * KW);
                        const uint4* m4 = reinterpret_cast<const uint4*>(row + NW + sub * KW);
#pragma unroll
                        for (int i = 0; i < KW / 2; ++i) {
                            const uint4 a = r4[i], c = m4[i];
                            pv[b][2 * i] = ((uint64_t)a.y << 32) | a.x; pv[b][2 * i + 1] = ((uint64_t)a.w << 32) | a.z;
                            sv[b][2 * i] = ((uint64_t)c.y << 32) | c.x; sv[b][2 * i + 1] = ((uint64_t)c.w << 32) | c.z;
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < KW; ++i) {
                            const int w = sub + i * G;
                            pv[b][i] = w < NW ? row[w] : 0ull;
                            sv[b][i] = w < NW ? row[NW + w] : 0ull;
                        }
                    }
                }
#pragma unroll
                for (int b = 0; b < BATCH; ++b)
#pragma unroll
                    for (int i = 0; i < KW; ++i) acc ^= pv[b][i] ^ sv[b][i];
            }
        }
    } else {
        const int sub = lane & 3, grp = lane >> 2;
        for (int64_t base = (int64_t)blockIdx.x * 64; base + 64 <= n_ids; base += (int64_t)gridDim.x * 64) {
            const uint32_t mine = ids[base + lane];
            for (int w0 = sub; w0 < row_words; w0 += 24) {
                uint64_t t[4][6];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t row = (uint32_t)__shfl((int)mine, b * 16 + grp);
                    const uint64_t* p = codes + (int64_t)row * row_words;
#pragma unroll
                    for (int u = 0; u < 6; ++u) t[b][u] = w0 + 4 * u < row_words ? p[w0 + 4 * u] : 0ull;
                }
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int u = 0; u < 6; ++u) acc ^= t[b][u];
            }
        }
    }
    if (acc == 0x0123456789ABCDEFull) sink[0] = acc;  // keeps the loads alive
}

// Copies dense code rows (planes of nw words) into rows `stride` words apart whose planes are plane_words long;
// everything that is not a code word is zero.  One thread per output word.
__global__ __launch_bounds__(256) void pad_codes_kernel(const uint64_t* __restrict__ codes, int64_t n, int nw, int planes,
                                                        int plane_words, int stride, uint64_t* __restrict__ out) {
    const int64_t total = n * stride;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / stride;
        const int at = (int)(i - row * stride);
        const int plane = at / plane_words, w = at - plane * plane_words;
        out[i] = (plane < planes && w < nw) ? codes[row * (planes * nw) + plane * nw + w] : 0ull;
    }
}

// Dense Sign-Magnitude rows (nw sign words, nw magnitude words) -> the two arrays of the split layout (kernels.h):
// out1 rows of split_stride1(nw) words = sign plane, first split_k1(nw) magnitude words, zeros; out2 rows of the remaining
// magnitude words.  One thread per input word.
__global__ __launch_bounds__(256) void split_codes_kernel(const uint64_t* __restrict__ codes, int64_t n, int nw,
                                                          uint64_t* __restrict__ out1, uint64_t* __restrict__ out2) {
    const int s1 = split_stride1(nw), k1 = split_k1(nw), s2 = split_stride2(nw);
    const int64_t total = n * s1 + n * s2;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        if (i < n * s1) {
            const int64_t row = i / s1;
            const int at = (int)(i - row * s1);
            out1[i] = at < nw + k1 ? codes[row * 2 * nw + at] : 0ull;    // sign words and the first magnitude words are contiguous
        } else {
            const int64_t j = i - n * s1, row = j / s2;
            const int at = (int)(j - row * s2);
            out2[j] = codes[row * 2 * nw + nw + k1 + at];
        }
    }
}

hipError_t launch_split_codes(const uint64_t* codes, int64_t n, int nw, uint64_t* out1, uint64_t* out2, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    int64_t blocks = (n * 2 * nw + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(split_codes_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, codes, n, nw, out1, out2);
    return hipGetLastError();
}

hipError_t launch_pad_codes(const uint64_t* codes, int64_t n, int nw, int planes, int plane_words, int stride, uint64_t* out,
                            hipStream_t stream) {
    if (n == 0) return hipSuccess;
    int64_t blocks = (n * stride + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(pad_codes_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, codes, n, nw, planes, plane_words, stride, out);
    return hipGetLastError();
}

hipError_t launch_gather_probe(const uint64_t* codes, int d, const uint32_t* ids, int64_t n_ids, uint64_t* sink,
                               hipStream_t stream) {
    if (n_ids < 64) return hipSuccess;
    int64_t blocks = n_ids / 64;
    if (blocks > 256 * 40) blocks = 256 * 40;
    const int nw = (d + 63) / 64;
    const dim3 grid((unsigned)blocks), block(64);
    switch (nw) {   // the widths of the workloads, with the lanes per row the search kernel picks for them
#define QV_PROBE(W, G) case W: hipLaunchKernelGGL((gather_probe_kernel<W, G>), grid, block, 0, stream, codes, 2 * nw, ids, n_ids, sink); break;
        QV_PROBE(2, 2) QV_PROBE(4, 2) QV_PROBE(6, 2) QV_PROBE(8, 2) QV_PROBE(12, 2) QV_PROBE(16, 4) QV_PROBE(24, 4)
        QV_PROBE(32, 4) QV_PROBE(48, 16)
#undef QV_PROBE
        default: hipLaunchKernelGGL((gather_probe_kernel<0, 4>), grid, block, 0, stream, codes, 2 * nw, ids, n_ids, sink);
    }
    return hipGetLastError();
}

hipError_t launch_encode(const float* x, int64_t n, int d, int encoding, uint64_t* codes, uint32_t* status,
                         hipStream_t stream) {
    if (n == 0) return hipSuccess;
    dim3 grid((unsigned)((n + ENC_WAVES - 1) / ENC_WAVES)), block(64 * ENC_WAVES);   // one vector per wave; n <= 2^32 (checked by the caller)
    auto grid_for = [&](int rows) { return dim3((unsigned)((n + ENC_WAVES * rows - 1) / (ENC_WAVES * rows))); };
    if (encoding == ENC_SIGN1) {
        hipLaunchKernelGGL(encode_sign1_kernel, grid, block, 0, stream, x, n, d, codes, status);
        return hipGetLastError();
    }
    if (encoding == ENC_SQ2) {   // the Sign-Magnitude decisions first, then their rewrite into levels
        hipError_t e = launch_encode(x, n, d, ENC_SM, codes, status, stream);
        if (e != hipSuccess) return e;
        int64_t blocks = (n * ((d + 63) / 64) + 255) / 256;
        if (blocks > 256 * 64) blocks = 256 * 64;
        hipLaunchKernelGGL(sq2_from_sm_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, codes, n, d);
        return hipGetLastError();
    }
    // vectors per wave, measured at 1M vectors: 64 x W dimensions of 4 (256-d: 0.168 against 0.191 ms with one) and
    // 6 words (384-d with two: 0.263 against 0.300 ms) gain; from 8 words on one vector per wave is as fast
    switch ((d + 63) / 64) {
#define QV_ENC_CASE(W, ROWS) case W: hipLaunchKernelGGL((encode_kernel_reg<W, ROWS>), grid_for(ROWS), block, 0, stream, x, n, d, codes, status); break;
        QV_ENC_CASE(1, 8) QV_ENC_CASE(2, 4) QV_ENC_CASE(3, 4) QV_ENC_CASE(4, 4) QV_ENC_CASE(5, 2) QV_ENC_CASE(6, 2)
        QV_ENC_CASE(7, 1) QV_ENC_CASE(8, 1) QV_ENC_CASE(9, 1) QV_ENC_CASE(10, 1) QV_ENC_CASE(11, 1) QV_ENC_CASE(12, 1)
        QV_ENC_CASE(13, 1) QV_ENC_CASE(14, 1) QV_ENC_CASE(15, 1) QV_ENC_CASE(16, 1) QV_ENC_CASE(17, 1) QV_ENC_CASE(18, 1)
        QV_ENC_CASE(19, 1) QV_ENC_CASE(20, 1) QV_ENC_CASE(21, 1) QV_ENC_CASE(22, 1) QV_ENC_CASE(23, 1) QV_ENC_CASE(24, 1)
        QV_ENC_CASE(32, 1) QV_ENC_CASE(48, 1) QV_ENC_CASE(64, 1)
#undef QV_ENC_CASE
        default: hipLaunchKernelGGL(encode_kernel, grid, block, 0, stream, x, n, d, codes, status);
    }
    return hipGetLastError();
}

hipError_t launch_bq_distance(const uint64_t* a, const int64_t* ia, const uint64_t* b, const int64_t* ib,
                              int64_t npairs, int d, int encoding, uint32_t* out, hipStream_t stream) {
    if (npairs == 0) return hipSuccess;
    int W = (d + 63) / 64;
    dim3 grid((unsigned)((npairs + 255) / 256));
    hipLaunchKernelGGL(bq_distance_kernel, grid, dim3(256), 0, stream, a, ia, b, ib, npairs, W, encoding, out);
    return hipGetLastError();
}

}  // namespace qv
