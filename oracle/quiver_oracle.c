/*
 * quiver_oracle.c -- plain CPU oracle for the QuIVer query hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines, in the most direct way we
 * could write it, what the GPU library must compute.  It is slow on purpose:
 * no popcount tricks, no SIMD, no blocking, no fusion.  It shares no code,
 * header, table or helper with the HIP library, and nothing in the product
 * path may call it.  Only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg load it.
 *
 * What it follows in the paper (arxiv 2605.02171):
 *   - Sec. 3.1, the two unnumbered encoding equations: tau = mean |x_i|,
 *     pos_i = [x_i > 0], strong_i = [|x_i| > tau].
 *   - Sec. 3.1 "Symmetric distance", Table 1: a dimension costs 0 when the
 *     signs agree and 4 / 2 / 1 when they differ and both / one / none of the
 *     two magnitude bits are set.
 *   - Sec. 3.3 Stage 1: greedy best-first beam search over the graph with an
 *     ef-wide candidate list, navigating with the symmetric distance only.
 *   - Sec. 3.3 Stage 2: the final candidates are re-scored with the exact
 *     cosine similarity against the float32 query, best k returned.
 *
 * Readings taken where the paper is silent (each one is a decision of this
 * build, not of the paper):
 *   - "mean" is the exact real-number mean: strong_i <=> D*|x_i| > sum_j |x_j|
 *     evaluated without any rounding (big-integer arithmetic below).
 *   - both tests are strict; +0.0 and -0.0 are "not positive".
 *   - packing: W = ceil(D/64) 64-bit words of sign bits followed by W words of
 *     magnitude bits; dimension i lives in word i/64, bit i%64 (bit 0 = LSB);
 *     bits of dimensions >= D are zero.
 *   - beam search: one sorted list keyed by (distance, id), smaller id wins a
 *     tie; a node is marked visited when its distance is first computed; the
 *     search stops when the list holds no unexpanded entry.
 *   - rerank: all entries of the final list, cosine accumulated in double,
 *     rounded to float once, ordered by (score descending, id ascending).
 *
 *
 * The two alternative encodings of the paper's ablation (Sec. 5.5 "Encoding
 * Ablation", Table 10) are here as well, selected by an `enc` argument of the
 * *_enc entry points (0 = Sign-Magnitude, the default everywhere else):
 *   - enc 1, "1-bit sign": pos_i only, distance = number of differing signs.
 *   - enc 2, "2-bit SQ": every dimension falls into one of four equal-width
 *     buckets, distance = sum of |level_a - level_b| (L1).  The paper does not
 *     say over which range; the reading here is the vector's own value range
 *     [min_i x_i, max_i x_i] (so no training data is involved, like tau):
 *     level = number of k in {1,2,3} with 4*(x - min) >= k*(max - min), every
 *     product and difference evaluated in IEEE double in exactly this form; a
 *     constant vector gets level 3 everywhere.  Stored as two bit-planes, low
 *     bit of the level first, same packing as above.
 *
 * Parity pins for every function here live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_NONFINITE (-2)
#define ORC_ERR_NOMEM (-3)

#define ORC_EMPTY 0xFFFFFFFFu

/* ------------------------------------------------------------------ */
/* Exact arithmetic on |float| values.                                 */
/* A finite float |x| equals M * 2^(o-149) with integers M < 2^24 and  */
/* 0 <= o <= 253.  Sums of such numbers are held as little-endian      */
/* base-2^32 integers in units of 2^-149.                              */
/* ------------------------------------------------------------------ */
#define BIG_WORDS 12 /* 384 bits: 253 + 24 + 32 (count) + 32 (factor D) fit */

typedef struct {
    uint32_t w[BIG_WORDS];
} big_t;

static void big_zero(big_t *a) { memset(a->w, 0, sizeof(a->w)); }

/* a += m * 2^sh, with m < 2^62 and sh <= 253 */
static void big_add_shifted(big_t *a, uint64_t m, int sh) {
    int word = sh / 32;
    int bit = sh % 32;
    unsigned __int128 v = (unsigned __int128)m << bit; /* < 2^94 */
    uint64_t carry = 0;
    for (int k = word; k < BIG_WORDS; ++k) {
        uint64_t piece = (uint64_t)(v & 0xFFFFFFFFu);
        v >>= 32;
        uint64_t s = (uint64_t)a->w[k] + piece + carry;
        a->w[k] = (uint32_t)s;
        carry = s >> 32;
        if (v == 0 && carry == 0) break;
    }
}

/* sign of (a - b): -1, 0, +1 */
static int big_cmp(const big_t *a, const big_t *b) {
    for (int k = BIG_WORDS - 1; k >= 0; --k) {
        if (a->w[k] > b->w[k]) return 1;
        if (a->w[k] < b->w[k]) return -1;
    }
    return 0;
}

/* split |x| into integer mantissa and shift; returns 0 for non-finite */
static int split_abs(float x, uint32_t *mant, int *shift) {
    uint32_t u;
    memcpy(&u, &x, 4);
    uint32_t e = (u >> 23) & 0xFFu;
    uint32_t f = u & 0x7FFFFFu;
    if (e == 0xFFu) return 0;
    if (e == 0) {
        *mant = f;
        *shift = 0;
    } else {
        *mant = f | 0x800000u;
        *shift = (int)e - 1;
    }
    return 1;
}

int orc_code_words(int d) { return d < 1 ? 0 : 2 * ((d + 63) / 64); }

/*
 * Encode one vector (Sec. 3.1 encoding equations).
 * code: 2*W words, written in full.
 */
static int encode_one(const float *x, int d, uint64_t *code) {
    int W = (d + 63) / 64;
    big_t S;
    big_zero(&S);
    for (int i = 0; i < d; ++i) {
        uint32_t m;
        int sh;
        if (!split_abs(x[i], &m, &sh)) return ORC_ERR_NONFINITE;
        big_add_shifted(&S, m, sh); /* S = sum_j |x_j|, exact */
    }
    for (int w = 0; w < 2 * W; ++w) code[w] = 0;
    for (int i = 0; i < d; ++i) {
        uint32_t m = 0;
        int sh = 0;
        split_abs(x[i], &m, &sh);
        /* strong_i <=> |x_i| > S/D  <=>  D*|x_i| > S */
        big_t T;
        big_zero(&T);
        big_add_shifted(&T, (uint64_t)m * (uint64_t)d, sh);
        int strong = big_cmp(&T, &S) > 0;
        int pos = x[i] > 0.0f;
        if (pos) code[i / 64] |= (uint64_t)1 << (i % 64);
        if (strong) code[W + i / 64] |= (uint64_t)1 << (i % 64);
    }
    return ORC_OK;
}

/* x[n][d] row-major -> codes[n][2W].  Vectors are independent. */
int orc_encode(const float *x, int64_t n, int d, uint64_t *codes, int threads) {
    if (!x || !codes || n < 0 || d < 1) return ORC_ERR_ARG;
    int cw = orc_code_words(d);
    int rc = ORC_OK;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(static) num_threads(threads)
    for (int64_t v = 0; v < n; ++v) {
        int r = encode_one(x + v * (int64_t)d, d, codes + v * (int64_t)cw);
        if (r != ORC_OK) {
#pragma omp critical
            rc = r;
        }
    }
    return rc;
}

/* ------------------------------------------------------------------ */
/* Symmetric Sign-Magnitude distance (Sec. 3.1, Table 1).              */
/* Walks the dimensions one by one and looks the penalty up.           */
/* ------------------------------------------------------------------ */
static const uint32_t PENALTY_DIFFERENT_SIGN[2][2] = {
    /* b weak, b strong */
    {1u, 2u}, /* a weak   */
    {2u, 4u}, /* a strong */
};

static int code_bit(const uint64_t *plane, int i) { return (int)((plane[i / 64] >> (i % 64)) & 1u); }

uint32_t orc_sm_distance(const uint64_t *a, const uint64_t *b, int d) {
    int W = (d + 63) / 64;
    uint32_t dist = 0;
    for (int i = 0; i < d; ++i) {
        int pa = code_bit(a, i), pb = code_bit(b, i);
        int sa = code_bit(a + W, i), sb = code_bit(b + W, i);
        if (pa != pb) dist += PENALTY_DIFFERENT_SIGN[sa][sb];
        /* same sign: contributes 0 whatever the magnitude bits are */
    }
    return dist;
}

/* pairs: out[p] = dist(codes_a[ia[p]], codes_b[ib[p]]) */
int orc_sm_distance_pairs(const uint64_t *codes_a, const int64_t *ia, const uint64_t *codes_b, const int64_t *ib,
                          int64_t npairs, int d, uint32_t *out) {
    if (!codes_a || !codes_b || !ia || !ib || !out || d < 1 || npairs < 0) return ORC_ERR_ARG;
    int cw = orc_code_words(d);
    for (int64_t p = 0; p < npairs; ++p)
        out[p] = orc_sm_distance(codes_a + ia[p] * (int64_t)cw, codes_b + ib[p] * (int64_t)cw, d);
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Ablation encodings (Sec. 5.5, Table 10).                            */
/* ------------------------------------------------------------------ */
#define ORC_ENC_SM 0
#define ORC_ENC_SIGN1 1
#define ORC_ENC_SQ2 2

int orc_code_words_enc(int d, int enc) {
    if (d < 1 || enc < 0 || enc > 2) return 0;
    return (enc == ORC_ENC_SIGN1 ? 1 : 2) * ((d + 63) / 64);
}

static int encode_sign1(const float *x, int d, uint64_t *code) {
    int W = (d + 63) / 64;
    for (int w = 0; w < W; ++w) code[w] = 0;
    for (int i = 0; i < d; ++i) {
        if (!isfinite(x[i])) return ORC_ERR_NONFINITE;
        if (x[i] > 0.0f) code[i / 64] |= (uint64_t)1 << (i % 64);
    }
    return ORC_OK;
}

/*
 * 2-bit uniform scalar quantiser of the ablation (Sec. 5.5: "four equal-width buckets", L1 distance on the bucket
 * indices).  The paper does not say which range the buckets divide.  Reading taken: like the method's own
 * threshold, the range comes from the vector itself and needs no training data: [-2 tau, +2 tau] with tau the exact
 * mean magnitude, i.e. bucket edges at -tau, 0, +tau, values beyond the range falling into the outer buckets.
 * (With this range the quantiser ranks slightly better than the Sign-Magnitude code and both clearly better than the
 * sign alone -- the order Table 10 reports; a range of [min, max] of the vector ranks worse than the sign alone.)
 * An element equal to an edge goes with the tests of Sec. 3.1, which are strict: level 3 iff x > tau, level 2 iff
 * 0 < x <= tau, level 1 iff -tau <= x <= 0, level 0 iff x < -tau.
 * Planes: low bit of the level, then high bit.
 */
static int encode_sq2(const float *x, int d, uint64_t *code) {
    int W = (d + 63) / 64;
    big_t S;
    big_zero(&S);
    for (int i = 0; i < d; ++i) {
        uint32_t m;
        int sh;
        if (!split_abs(x[i], &m, &sh)) return ORC_ERR_NONFINITE;
        big_add_shifted(&S, m, sh); /* S = sum_j |x_j| = D * tau, exact */
    }
    for (int w = 0; w < 2 * W; ++w) code[w] = 0;
    for (int i = 0; i < d; ++i) {
        uint32_t m = 0;
        int sh = 0;
        split_abs(x[i], &m, &sh);
        big_t T; /* D * |x_i| */
        big_zero(&T);
        big_add_shifted(&T, (uint64_t)m * (uint64_t)d, sh);
        int beyond = big_cmp(&T, &S) > 0; /* |x_i| > tau */
        int level;
        if (x[i] > 0.0f) level = beyond ? 3 : 2;
        else level = beyond ? 0 : 1;
        if (level & 1) code[i / 64] |= (uint64_t)1 << (i % 64);
        if (level & 2) code[W + i / 64] |= (uint64_t)1 << (i % 64);
    }
    return ORC_OK;
}

static int encode_vec(int enc, const float *x, int d, uint64_t *code) {
    if (enc == ORC_ENC_SIGN1) return encode_sign1(x, d, code);
    if (enc == ORC_ENC_SQ2) return encode_sq2(x, d, code);
    return encode_one(x, d, code);
}

int orc_encode_enc(const float *x, int64_t n, int d, int enc, uint64_t *codes, int threads) {
    if (!x || !codes || n < 0 || d < 1 || enc < 0 || enc > 2) return ORC_ERR_ARG;
    int cw = orc_code_words_enc(d, enc);
    int rc = ORC_OK;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(static) num_threads(threads)
    for (int64_t v = 0; v < n; ++v) {
        int r = encode_vec(enc, x + v * (int64_t)d, d, codes + v * (int64_t)cw);
        if (r != ORC_OK) {
#pragma omp critical
            rc = r;
        }
    }
    return rc;
}

/* distance of two codes of the same encoding, dimension by dimension */
uint32_t orc_distance_enc(const uint64_t *a, const uint64_t *b, int d, int enc) {
    if (enc == ORC_ENC_SM) return orc_sm_distance(a, b, d);
    int W = (d + 63) / 64;
    uint32_t dist = 0;
    for (int i = 0; i < d; ++i) {
        if (enc == ORC_ENC_SIGN1) {
            if (code_bit(a, i) != code_bit(b, i)) dist += 1u;
        } else {
            int la = code_bit(a, i) + 2 * code_bit(a + W, i);
            int lb = code_bit(b, i) + 2 * code_bit(b + W, i);
            dist += (uint32_t)(la > lb ? la - lb : lb - la);
        }
    }
    return dist;
}

int orc_distance_pairs_enc(const uint64_t *codes_a, const int64_t *ia, const uint64_t *codes_b, const int64_t *ib,
                           int64_t npairs, int d, int enc, uint32_t *out) {
    if (!codes_a || !codes_b || !ia || !ib || !out || d < 1 || npairs < 0 || enc < 0 || enc > 2) return ORC_ERR_ARG;
    int cw = orc_code_words_enc(d, enc);
    for (int64_t p = 0; p < npairs; ++p)
        out[p] = orc_distance_enc(codes_a + ia[p] * (int64_t)cw, codes_b + ib[p] * (int64_t)cw, d, enc);
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Stage 1: beam search (Sec. 3.3).                                    */
/* ------------------------------------------------------------------ */
typedef struct {
    uint32_t dist;
    uint32_t id;
    int expanded;
} entry_t;

static int key_less(uint32_t da, uint32_t ia, uint32_t db, uint32_t ib) {
    if (da != db) return da < db;
    return ia < ib;
}

/*
 * One query.  visited: n bytes, all zero on entry, all zero on return.
 * cand_id / cand_dist: ef slots (unused slots get ORC_EMPTY).
 * order: visit_cap slots (expanded ids in expansion order, rest ORC_EMPTY); may be NULL.
 * counters[0] = list length, [1] = nodes expanded, [2] = distances computed.
 */
static int beam_search_one(int enc, const uint64_t *qcode, int64_t n, int d, int R, const uint32_t *adj,
                           const uint64_t *codes, uint32_t entry, int ef, uint8_t *visited, entry_t *pool,
                           uint32_t *touched, uint32_t *cand_id, uint32_t *cand_dist, uint32_t *order,
                           int64_t visit_cap, uint32_t *counters) {
    int cw = orc_code_words_enc(d, enc);
    int size = 0;
    int64_t n_touched = 0;
    uint32_t n_evals = 0, n_expanded = 0;

    pool[0].dist = orc_distance_enc(qcode, codes + (int64_t)entry * cw, d, enc);
    pool[0].id = entry;
    pool[0].expanded = 0;
    size = 1;
    visited[entry] = 1;
    touched[n_touched++] = entry;
    n_evals = 1;

    for (;;) {
        int u = -1;
        for (int i = 0; i < size; ++i) {
            if (!pool[i].expanded) {
                u = i;
                break;
            }
        }
        if (u < 0) break;
        pool[u].expanded = 1;
        uint32_t uid = pool[u].id;
        if (order && (int64_t)n_expanded < visit_cap) order[n_expanded] = uid;
        n_expanded++;

        for (int j = 0; j < R; ++j) {
            uint32_t v = adj[(int64_t)uid * R + j];
            if (v == ORC_EMPTY) continue;
            if ((int64_t)v >= n) { /* malformed graph: undo the marks and give up */
                for (int64_t i = 0; i < n_touched; ++i) visited[touched[i]] = 0;
                return ORC_ERR_ARG;
            }
            if (visited[v]) continue;
            visited[v] = 1;
            touched[n_touched++] = v;
            uint32_t dv = orc_distance_enc(qcode, codes + (int64_t)v * cw, d, enc);
            n_evals++;
            if (size < ef || key_less(dv, v, pool[size - 1].dist, pool[size - 1].id)) {
                int p = size < ef ? size : ef - 1; /* slot that becomes free */
                while (p > 0 && key_less(dv, v, pool[p - 1].dist, pool[p - 1].id)) {
                    pool[p] = pool[p - 1];
                    --p;
                }
                pool[p].dist = dv;
                pool[p].id = v;
                pool[p].expanded = 0;
                if (size < ef) size++;
            }
        }
    }
    for (int i = 0; i < ef; ++i) {
        cand_id[i] = i < size ? pool[i].id : ORC_EMPTY;
        cand_dist[i] = i < size ? pool[i].dist : ORC_EMPTY;
    }
    if (order)
        for (int64_t i = n_expanded; i < visit_cap; ++i) order[i] = ORC_EMPTY;
    counters[0] = (uint32_t)size;
    counters[1] = n_expanded;
    counters[2] = n_evals;
    for (int64_t i = 0; i < n_touched; ++i) visited[touched[i]] = 0;
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Stage 2: float32 cosine rerank (Sec. 3.3).                          */
/* ------------------------------------------------------------------ */
static float cosine(const float *q, const float *x, int d) {
    double dot = 0.0, qq = 0.0, xx = 0.0;
    for (int i = 0; i < d; ++i) {
        dot += (double)q[i] * (double)x[i];
        qq += (double)q[i] * (double)q[i];
        xx += (double)x[i] * (double)x[i];
    }
    if (qq == 0.0 || xx == 0.0) return 0.0f;
    return (float)(dot / (sqrt(qq) * sqrt(xx)));
}

/* better: higher score first, then smaller id */
static int rank_before(float sa, uint32_t ia, float sb, uint32_t ib) {
    if (sa != sb) return sa > sb;
    return ia < ib;
}

static void rerank_one(const float *q, const float *vecs, int d, const uint32_t *cand_id, int n_cand, int k,
                       uint32_t *ids, float *scores, float *all_scores /* n_cand, may be NULL */) {
    float *s = (float *)malloc(sizeof(float) * (size_t)(n_cand > 0 ? n_cand : 1));
    uint32_t *o = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n_cand > 0 ? n_cand : 1));
    for (int c = 0; c < n_cand; ++c) {
        s[c] = cosine(q, vecs + (int64_t)cand_id[c] * d, d);
        if (all_scores) all_scores[c] = s[c];
        o[c] = (uint32_t)c;
    }
    /* insertion sort of the index array by (score desc, id asc) */
    for (int a = 1; a < n_cand; ++a) {
        uint32_t cur = o[a];
        int b = a;
        while (b > 0 && rank_before(s[cur], cand_id[cur], s[o[b - 1]], cand_id[o[b - 1]])) {
            o[b] = o[b - 1];
            --b;
        }
        o[b] = cur;
    }
    for (int r = 0; r < k; ++r) {
        if (r < n_cand) {
            ids[r] = cand_id[o[r]];
            scores[r] = s[o[r]];
        } else {
            ids[r] = ORC_EMPTY;
            scores[r] = -INFINITY;
        }
    }
    free(s);
    free(o);
}

/* Standalone rerank of given candidate lists: cand_id[nq][ef] (ORC_EMPTY padded, n_cand[nq]). */
int orc_rerank(const float *queries, int64_t nq, int d, const float *vecs, const uint32_t *cand_id, int ef,
               const uint32_t *n_cand, int k, uint32_t *ids, float *scores, float *all_scores) {
    if (!queries || !vecs || !cand_id || !n_cand || !ids || !scores || d < 1 || k < 1 || ef < k) return ORC_ERR_ARG;
    for (int64_t q = 0; q < nq; ++q)
        rerank_one(queries + q * d, vecs, d, cand_id + q * ef, (int)n_cand[q], k, ids + q * k, scores + q * k,
                   all_scores ? all_scores + q * ef : NULL);
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Whole path for a batch: encode query, beam search, rerank.          */
/* Queries are independent; `threads` > 1 only spreads them over cores. */
/* Optional outputs may be NULL.                                        */
/* ------------------------------------------------------------------ */
int orc_search_enc(int enc, const float *queries, int64_t nq, int64_t n, int d, int R, const uint32_t *adj,
               const uint64_t *codes, const float *vecs /* NULL: skip stage 2 */, uint32_t entry, int k, int ef,
               uint32_t *ids, float *scores,             /* [nq][k], NULL if vecs NULL */
               uint32_t *cand_id, uint32_t *cand_dist,   /* [nq][ef] */
               uint32_t *counters,                       /* [nq][3] */
               uint32_t *order, int64_t visit_cap,       /* [nq][visit_cap] or NULL */
               int threads) {
    if (!queries || !adj || !codes || !cand_id || !cand_dist || !counters || enc < 0 || enc > 2) return ORC_ERR_ARG;
    if (nq < 0 || n < 1 || d < 1 || R < 1 || ef < 1 || (int64_t)entry >= n) return ORC_ERR_ARG;
    if (vecs && (k < 1 || k > ef || !ids || !scores)) return ORC_ERR_ARG;
    if (threads < 1) threads = 1;
    int cw = orc_code_words_enc(d, enc);
    int rc = ORC_OK;
#pragma omp parallel num_threads(threads)
    {
        uint8_t *visited = (uint8_t *)calloc((size_t)n, 1);
        uint32_t *touched = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n);
        entry_t *pool = (entry_t *)malloc(sizeof(entry_t) * (size_t)(ef + 1));
        uint64_t *qcode = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)cw);
        int ok = visited && touched && pool && qcode;
        if (!ok) {
#pragma omp critical
            rc = ORC_ERR_NOMEM;
        }
#pragma omp for schedule(dynamic, 8)
        for (int64_t q = 0; q < nq; ++q) {
            if (!ok) continue;
            int r = encode_vec(enc, queries + q * d, d, qcode);
            if (r == ORC_OK)
                r = beam_search_one(enc, qcode, n, d, R, adj, codes, entry, ef, visited, pool, touched,
                                    cand_id + q * ef, cand_dist + q * ef, order ? order + q * visit_cap : NULL,
                                    visit_cap, counters + q * 3);
            if (r == ORC_OK && vecs)
                rerank_one(queries + q * d, vecs, d, cand_id + q * ef, (int)counters[q * 3], k, ids + q * k,
                           scores + q * k, NULL);
            if (r != ORC_OK) {
#pragma omp critical
                rc = r;
            }
        }
        free(visited);
        free(touched);
        free(pool);
        free(qcode);
    }
    return rc;
}

int orc_search(const float *queries, int64_t nq, int64_t n, int d, int R, const uint32_t *adj, const uint64_t *codes,
               const float *vecs, uint32_t entry, int k, int ef, uint32_t *ids, float *scores, uint32_t *cand_id,
               uint32_t *cand_dist, uint32_t *counters, uint32_t *order, int64_t visit_cap, int threads) {
    return orc_search_enc(ORC_ENC_SM, queries, nq, n, d, R, adj, codes, vecs, entry, k, ef, ids, scores, cand_id, cand_dist,
                          counters, order, visit_cap, threads);
}

/* ------------------------------------------------------------------ */
/* Brute-force scan in code space (Sec. 6 "Practical compatibility     */
/* test"; Sec. 5.5 Table 10 "Top-10 overlap"): for every query code    */
/* the K base codes with the smallest (distance, id), by computing     */
/* every distance.  ids/dist: [nq][K], ORC_EMPTY padded when n < K.    */
/* ------------------------------------------------------------------ */
int orc_bq_scan_enc(int enc, const uint64_t *codes, int64_t n, int d, const uint64_t *qcodes, int64_t nq, int K,
                    uint32_t *ids, uint32_t *dist, int threads) {
    if (!codes || !qcodes || !ids || !dist || n < 0 || nq < 0 || d < 1 || K < 1 || enc < 0 || enc > 2) return ORC_ERR_ARG;
    if (threads < 1) threads = 1;
    int cw = orc_code_words_enc(d, enc);
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int64_t q = 0; q < nq; ++q) {
        uint32_t *bi = ids + q * K, *bd = dist + q * K;
        int size = 0;
        for (int j = 0; j < K; ++j) bi[j] = bd[j] = ORC_EMPTY;
        for (int64_t v = 0; v < n; ++v) {
            uint32_t dv = orc_distance_enc(qcodes + q * cw, codes + v * cw, d, enc);
            if (size < K || key_less(dv, (uint32_t)v, bd[size - 1], bi[size - 1])) {
                int p = size < K ? size : K - 1;
                while (p > 0 && key_less(dv, (uint32_t)v, bd[p - 1], bi[p - 1])) {
                    bd[p] = bd[p - 1];
                    bi[p] = bi[p - 1];
                    --p;
                }
                bd[p] = dv;
                bi[p] = (uint32_t)v;
                if (size < K) size++;
            }
        }
    }
    return ORC_OK;
}

int orc_bq_scan(const uint64_t *codes, int64_t n, int d, const uint64_t *qcodes, int64_t nq, int K, uint32_t *ids,
                uint32_t *dist, int threads) {
    return orc_bq_scan_enc(ORC_ENC_SM, codes, n, d, qcodes, nq, K, ids, dist, threads);
}

/* Exact float32-data top-K by cosine (double accumulation), order (score desc, id asc): the other side of the
 * overlap probe.  ids: [nq][K], ORC_EMPTY padded. */
int orc_cosine_topk(const float *vecs, int64_t n, int d, const float *queries, int64_t nq, int K, uint32_t *ids,
                    int threads) {
    if (!vecs || !queries || !ids || n < 0 || nq < 0 || d < 1 || K < 1) return ORC_ERR_ARG;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int64_t q = 0; q < nq; ++q) {
        uint32_t *bi = ids + q * K;
        float *bs = (float *)malloc(sizeof(float) * (size_t)K);
        int size = 0;
        for (int j = 0; j < K; ++j) bi[j] = ORC_EMPTY;
        for (int64_t v = 0; v < n; ++v) {
            float s = cosine(queries + q * d, vecs + v * d, d);
            if (size < K || rank_before(s, (uint32_t)v, bs[size - 1], bi[size - 1])) {
                int p = size < K ? size : K - 1;
                while (p > 0 && rank_before(s, (uint32_t)v, bs[p - 1], bi[p - 1])) {
                    bs[p] = bs[p - 1];
                    bi[p] = bi[p - 1];
                    --p;
                }
                bs[p] = s;
                bi[p] = (uint32_t)v;
                if (size < K) size++;
            }
        }
        free(bs);
    }
    return ORC_OK;
}

/* Mean fraction of a[q][0..K) that also occurs in b[q][0..K) (ORC_EMPTY entries never match). */
double orc_topk_overlap(const uint32_t *a, const uint32_t *b, int64_t nq, int K) {
    if (!a || !b || nq < 1 || K < 1) return -1.0;
    int64_t hits = 0;
    for (int64_t q = 0; q < nq; ++q)
        for (int i = 0; i < K; ++i) {
            uint32_t x = a[q * K + i];
            if (x == ORC_EMPTY) continue;
            for (int j = 0; j < K; ++j)
                if (b[q * K + j] == x) {
                    hits++;
                    break;
                }
        }
    return (double)hits / (double)(nq * K);
}

/* ------------------------------------------------------------------ */
/* Graph construction in code space (Sec. 3.2, Algorithm 1 "BQ-Vamana  */
/* Edge Selection" with the bidirectional re-selection of Sec. 2.2).   */
/*                                                                     */
/* The paper inserts nodes concurrently under per-node locks (Sec. 4.1)*/
/* which has no single defined result.  The reading taken here is the  */
/* batch-synchronous one, whose result is a function of the inputs:    */
/*   nodes are inserted in id order, in batches of max(1, done/50)     */
/*   (at most max_batch); every node of a batch searches the graph as  */
/*   it stood before the batch (beam width L, from `entry`), takes as  */
/*   candidates the final list plus its current out-neighbours, and    */
/*   selects its out-edges by Algorithm 1; then every node b that was  */
/*   selected receives the selecting nodes as in-edge candidates: if   */
/*   they fit in the row they are added, otherwise the row is          */
/*   re-selected by Algorithm 1 from (old row U new candidates).       */
/*   A node considers at most ORC_MAX_NEW_IN_EDGES new candidates per  */
/*   batch: the nearest ones by (distance, id).  Only hub nodes that   */
/*   hundreds of batch members select at once ever reach that cap.     */
/* The order of ids inside a row carries no meaning (the search does   */
/* not depend on it); rows are compared as sets.                       */
/* ------------------------------------------------------------------ */
#define ORC_MAX_NEW_IN_EDGES 192

typedef struct {
    uint32_t dist;
    uint32_t id;
} cand_t;

static int cand_cmp(const void *a, const void *b) {
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->dist != y->dist) return x->dist < y->dist ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

/* Algorithm 1: cand sorted by (dist to t, id), without t and without repeats; returns |selected| */
static int select_edges(int enc, const uint64_t *codes, int cw, int d, const cand_t *cand, int n_cand, int R,
                        double alpha, uint32_t *selected) {
    int ns = 0;
    for (int i = 0; i < n_cand && ns < R; ++i) {
        int keep = 1;
        for (int j = 0; j < ns && keep; ++j) {
            uint32_t dcs = orc_distance_enc(codes + (int64_t)cand[i].id * cw, codes + (int64_t)selected[j] * cw, d, enc);
            if (!((double)cand[i].dist <= alpha * (double)dcs)) keep = 0;
        }
        if (keep) selected[ns++] = cand[i].id;
    }
    return ns;
}

int orc_build_graph_enc(int enc, const uint64_t *codes, int64_t n, int d, int R, int L, double alpha, uint32_t entry,
                        int64_t max_batch, uint32_t *adj) {
    if (!codes || !adj || n < 1 || d < 1 || R < 1 || L < 1 || alpha < 1.0 || (int64_t)entry >= n || max_batch < 1 ||
        enc < 0 || enc > 2)
        return ORC_ERR_ARG;
    int cw = orc_code_words_enc(d, enc);
    for (int64_t i = 0; i < n * R; ++i) adj[i] = ORC_EMPTY;
    uint8_t *visited = (uint8_t *)calloc((size_t)n, 1);
    uint32_t *touched = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n);
    entry_t *pool = (entry_t *)malloc(sizeof(entry_t) * (size_t)(L + 1));
    uint32_t *cid = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)L);
    uint32_t *cds = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)L);
    uint32_t counters[3];
    int64_t done = 0;
    int rc = ORC_OK;
    while (done < n && rc == ORC_OK) {
        int64_t bs = done / 50;
        if (bs < 1) bs = 1;
        if (bs > max_batch) bs = max_batch;
        if (done + bs > n) bs = n - done;
        uint32_t *fwd = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(bs * R));
        int *nfwd = (int *)malloc(sizeof(int) * (size_t)bs);
        /* 1. searches and selections against the graph as it stands */
        for (int64_t i = 0; i < bs && rc == ORC_OK; ++i) {
            uint32_t t = (uint32_t)(done + i);
            rc = beam_search_one(enc, codes + (int64_t)t * cw, n, d, R, adj, codes, entry, L, visited, pool, touched, cid,
                                 cds, NULL, 0, counters);
            if (rc != ORC_OK) break;
            cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(L + R));
            int nc = 0;
            for (int j = 0; j < (int)counters[0]; ++j)
                if (cid[j] != t) {
                    cand[nc].dist = cds[j];
                    cand[nc++].id = cid[j];
                }
            for (int j = 0; j < R; ++j) {
                uint32_t v = adj[(int64_t)t * R + j];
                if (v == ORC_EMPTY || v == t) continue;
                int have = 0;
                for (int k = 0; k < nc; ++k) have |= cand[k].id == v;
                if (!have) {
                    cand[nc].dist = orc_distance_enc(codes + (int64_t)t * cw, codes + (int64_t)v * cw, d, enc);
                    cand[nc++].id = v;
                }
            }
            qsort(cand, (size_t)nc, sizeof(cand_t), cand_cmp);
            nfwd[i] = select_edges(enc, codes, cw, d, cand, nc, R, alpha, fwd + i * R);
            free(cand);
        }
        /* 2. publish the rows of the batch */
        for (int64_t i = 0; i < bs && rc == ORC_OK; ++i)
            for (int j = 0; j < R; ++j) adj[(done + i) * R + j] = j < nfwd[i] ? fwd[i * R + j] : ORC_EMPTY;
        /* 3. in-edges: for every target, all nodes of the batch that selected it.
         *    The (target, source) pairs are sorted so that each target's sources sit together. */
        int64_t n_pairs = 0;
        for (int64_t i = 0; i < bs; ++i) n_pairs += nfwd[i];
        cand_t *pairs = (cand_t *)malloc(sizeof(cand_t) * (size_t)(n_pairs > 0 ? n_pairs : 1));
        n_pairs = 0;
        for (int64_t i = 0; i < bs; ++i)
            for (int j = 0; j < nfwd[i]; ++j) {
                pairs[n_pairs].dist = fwd[i * R + j];          /* target (sort key) */
                pairs[n_pairs++].id = (uint32_t)(done + i);    /* source */
            }
        qsort(pairs, (size_t)n_pairs, sizeof(cand_t), cand_cmp);
        for (int64_t p0 = 0; p0 < n_pairs && rc == ORC_OK;) {
            int64_t b = pairs[p0].dist, p1 = p0;
            while (p1 < n_pairs && pairs[p1].dist == (uint32_t)b) p1++;
            cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(R + (p1 - p0)));
            int nc = 0, deg, n_new = 0;
            for (int j = 0; j < R; ++j) {
                uint32_t v = adj[b * R + j];
                if (v == ORC_EMPTY) continue;
                cand[nc].id = v;
                cand[nc++].dist = orc_distance_enc(codes + b * cw, codes + (int64_t)v * cw, d, enc);
            }
            deg = nc;
            for (int64_t p = p0; p < p1; ++p) {
                uint32_t t = pairs[p].id;
                int have = t == (uint32_t)b;
                for (int k = 0; k < deg; ++k) have |= cand[k].id == t;
                if (have) continue;
                cand[nc].id = t;
                cand[nc++].dist = orc_distance_enc(codes + b * cw, codes + (int64_t)t * cw, d, enc);
                n_new++;
            }
            if (n_new > ORC_MAX_NEW_IN_EDGES) { /* keep the nearest new candidates only */
                qsort(cand + deg, (size_t)n_new, sizeof(cand_t), cand_cmp);
                n_new = ORC_MAX_NEW_IN_EDGES;
                nc = deg + n_new;
            }
            if (n_new > 0) {
                if (deg + n_new <= R) {
                    int slot = 0;
                    for (int k = deg; k < nc; ++k) {
                        while (adj[b * R + slot] != ORC_EMPTY) slot++;
                        adj[b * R + slot] = cand[k].id;
                    }
                } else {
                    uint32_t *sel = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)R);
                    qsort(cand, (size_t)nc, sizeof(cand_t), cand_cmp);
                    int ns = select_edges(enc, codes, cw, d, cand, nc, R, alpha, sel);
                    for (int j = 0; j < R; ++j) adj[b * R + j] = j < ns ? sel[j] : ORC_EMPTY;
                    free(sel);
                }
            }
            free(cand);
            p0 = p1;
        }
        free(pairs);
        free(fwd);
        free(nfwd);
        done += bs;
    }
    free(visited);
    free(touched);
    free(pool);
    free(cid);
    free(cds);
    return rc;
}

int orc_build_graph(const uint64_t *codes, int64_t n, int d, int R, int L, double alpha, uint32_t entry,
                    int64_t max_batch, uint32_t *adj) {
    return orc_build_graph_enc(ORC_ENC_SM, codes, n, d, R, L, alpha, entry, max_batch, adj);
}
