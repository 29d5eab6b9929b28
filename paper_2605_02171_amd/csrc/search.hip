// Stage 1 of the query path (paper Sec. 3.3): greedy best-first beam search over a fixed-degree
// graph, navigating only with the symmetric Sign-Magnitude distance of Sec. 3.1 / Table 1.
//
// Mapping to gfx950: one 64-lane wavefront per query, one wavefront per workgroup.
//   * candidate list ("pool"): ef sorted 64-bit keys held in registers, entry e in lane e%64,
//     register e/64.  key = dist << 33 | id << 1 | expanded, so integer order is (dist, id) order.
//   * visited set: bucketed table of ids in LDS (one 16-byte bucket per probe; 16-bit tags that identify
//     an id exactly, or 32-bit ids).  By default it is a small cache in which new ids displace old ones,
//     so that 16 queries fit a compute unit (16-bit tags: seven per bucket, placed in turn by a counter
//     in the bucket that one LDS atomic add advances, no retry); a forgotten node that comes up again is
//     evaluated again, which cannot change the list (see merge_new_keys) and is reported in the status
//     word.  The other mode never forgets (slots claimed by LDS compare-and-swap) and stops taking ids
//     when nearly full.
//   * expansion: lane j reads adj[u][j] (one coalesced row; the row of the runner-up is loaded one
//     expansion ahead), lanes filter their ids through the visited table, survivors are compacted
//     into LDS, then G lanes cooperate on one neighbour's code: lane s of a group loads words s,
//     s+G, ... of both bit-planes (8*G contiguous bytes per group per load instruction); all loads
//     of an expansion are issued before the first popcount.  XOR/AND/OR + popcount per lane, then
//     a reduce-scatter over the G lanes leaves each lane with the distance of one neighbour.
//   * merge: every new key below the current worst gets its final position from two counts (pool
//     keys below it, new keys below it), every pool key moves up by the number of new keys below
//     it, and one scatter through LDS puts everything in place.  The pool after an expansion is
//     the ef smallest keys of (old pool U new keys); that set does not depend on the order in
//     which neighbours are considered, so expanding all neighbours at once reproduces the
//     sequential algorithm exactly.
//   * launch order: workgroup b runs query order[b]; batches of 4,096 queries and more start their
//     probably-longest queries first (query_order_kernel).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "kernels.h"

namespace qv {

constexpr uint64_t KEY_NONE = ~0ull;

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ uint64_t readlane64(uint64_t v, int l) {
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}

// value of the lane whose index differs in bit 0 / bit 1 (data-parallel primitive, no LDS traffic)
__device__ __forceinline__ uint32_t quad_xor1(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);  // quad_perm:[1,0,3,2]
}
__device__ __forceinline__ uint32_t quad_xor2(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);  // quad_perm:[2,3,0,1]
}

// Per 64 dimensions (Table 1 of the paper as three popcounts): with X = differing signs,
// c1 += pc(X), c2 += pc(X and (s_v or s_q)), c3 += pc(X and s_v and s_q); distance = c1 + c2 + 2*c3.
// The two masked terms are single three-input bit operations on gfx950 (truth tables 0xE0 = a&(b|c),
// 0x80 = a&b&c with a = 0xF0, b = 0xCC, c = 0xAA).
// popcount(x) + acc in one instruction (the bit-count instruction has an addend; written out because the compiler
// otherwise counts into fresh registers and sums them with three-input adds, half as many instructions again)
__device__ __forceinline__ uint32_t popc_add(uint32_t x, uint32_t acc) {
    uint32_t r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
    return r;
}

__device__ __forceinline__ void sm_accumulate(uint64_t pv, uint64_t sv, uint64_t pq, uint64_t sq, uint32_t& c1,
                                              uint32_t& c2, uint32_t& c3) {
    const uint32_t xl = (uint32_t)pv ^ (uint32_t)pq, xh = (uint32_t)(pv >> 32) ^ (uint32_t)(pq >> 32);
    const uint32_t svl = (uint32_t)sv, svh = (uint32_t)(sv >> 32), sql = (uint32_t)sq, sqh = (uint32_t)(sq >> 32);
    c1 = popc_add(xh, popc_add(xl, c1));
    c2 = popc_add(__builtin_amdgcn_bitop3_b32(xh, svh, sqh, 0xE0), popc_add(__builtin_amdgcn_bitop3_b32(xl, svl, sql, 0xE0), c2));
    c3 = popc_add(__builtin_amdgcn_bitop3_b32(xh, svh, sqh, 0x80), popc_add(__builtin_amdgcn_bitop3_b32(xl, svl, sql, 0x80), c3));
}

// The same step for any of the three encodings (ENC_SM: the method; ENC_SIGN1, ENC_SQ2: the two of the
// paper's ablation, Sec. 5.5 / Table 10).  w0, w1: the node's first and second bit-plane word; q0, q1,
// q2: the query's words as code_query_words() prepared them.
//   ENC_SIGN1  distance = pc(sign_v xor sign_q)                                  (w1, q1, q2 unused)
//   ENC_SQ2    level = 2*hi + lo; |level_v - level_q| = sum over k = 1..3 of [level_v >= k] xor [level_q >= k];
//              [level >= 1] = hi|lo, [level >= 2] = hi, [level >= 3] = hi&lo.  With w0 = lo, w1 = hi and
//              q0 = (hi|lo)_q, q1 = hi_q, q2 = (hi&lo)_q: three popcounts, the first and third of a single
//              three-input operation each (truth tables 0x56 = (a|b)^c, 0x6A = (a&b)^c).
template <int ENC>
__device__ __forceinline__ void code_accumulate(uint64_t w0, uint64_t w1, uint64_t q0, uint64_t q1, uint64_t q2,
                                                uint32_t& c1, uint32_t& c2, uint32_t& c3) {
    if constexpr (ENC == ENC_SM) {
        sm_accumulate(w0, w1, q0, q1, c1, c2, c3);
    } else if constexpr (ENC == ENC_SIGN1) {
        c1 += __popcll(w0 ^ q0);
    } else {
        const uint32_t ll = (uint32_t)w0, lh = (uint32_t)(w0 >> 32), hl = (uint32_t)w1, hh = (uint32_t)(w1 >> 32);
        c1 += __popc(__builtin_amdgcn_bitop3_b32(hl, ll, (uint32_t)q0, 0x56)) +
              __popc(__builtin_amdgcn_bitop3_b32(hh, lh, (uint32_t)(q0 >> 32), 0x56));
        c2 += __popcll(w1 ^ q1);
        c3 += __popc(__builtin_amdgcn_bitop3_b32(hl, ll, (uint32_t)q2, 0x6A)) +
              __popc(__builtin_amdgcn_bitop3_b32(hh, lh, (uint32_t)(q2 >> 32), 0x6A));
    }
}

template <int ENC>
__device__ __forceinline__ uint32_t code_distance_from_counts(uint32_t c1, uint32_t c2, uint32_t c3) {
    return ENC == ENC_SM ? c1 + c2 + 2u * c3 : c1 + c2 + c3;
}

// query words as code_accumulate() wants them, from the two plane words of the query's own code
template <int ENC>
__device__ __forceinline__ void code_query_words(uint64_t a, uint64_t b, uint64_t& q0, uint64_t& q1, uint64_t& q2) {
    if constexpr (ENC == ENC_SQ2) {
        q0 = a | b; q1 = b; q2 = a & b;
    } else {
        q0 = a; q1 = b; q2 = 0;
    }
}

// ---------------------------------------------------------------------------------------------
// Visited set, 32-bit entries: buckets of four ids; an id lives in the first bucket, counting from
// its home bucket, that had a free slot when it arrived.  Slots are never freed, so a lookup may
// stop at the first bucket that still has a free slot.
// Returns true when v was not in the table (and is now, if may_insert).
__device__ __forceinline__ bool visited32_test_and_set(uint32_t* tab, uint32_t bucket_mask, int bucket_bits,
                                                       uint32_t v, bool may_insert) {
    uint32_t b = (v * 2654435761u) >> (32 - bucket_bits);
    for (;;) {
        uint32_t* bp = tab + b * 4;
        const uint4 s = *reinterpret_cast<const uint4*>(bp);
        if (s.x == v || s.y == v || s.z == v || s.w == v) return false;
        const int e = s.x == EMPTY_ID ? 0 : (s.y == EMPTY_ID ? 1 : (s.z == EMPTY_ID ? 2 : (s.w == EMPTY_ID ? 3 : -1)));
        if (e < 0) {
            b = (b + 1) & bucket_mask;  // the table is never allowed to fill up, so this ends
            continue;
        }
        if (!may_insert) return true;
        const uint32_t old = atomicCAS(bp + e, EMPTY_ID, v);
        if (old == EMPTY_ID) return true;
        if (old == v) return false;     // another lane holds the same id and was first
        // another id took the slot: look at this bucket again
    }
}

// Visited set, 16-bit entries, for graphs of up to a few million nodes (half the LDS per query).
// An id is split as v = r0 * 65535 + t0; the table is cut into `regions` equal parts of B buckets,
// v lives in part (r0 + g(t0)) mod regions (g spreads consecutive ids over the parts) and stores
// only the tag t0 < 65535, so (part, tag) identifies v exactly; 0xFFFF = free.  Buckets hold eight
// tags (16 bytes); probing runs over the buckets of the part.  `failed` is raised when the part has
// no room left.
__device__ __forceinline__ uint32_t any_zero_half(uint32_t x) { return (x - 0x00010001u) & ~x & 0x80008000u; }

__device__ __forceinline__ bool visited16_test_and_set(uint32_t* tab32, uint32_t regions, uint32_t B, uint32_t v,
                                                       bool may_insert, bool& failed) {
    const uint32_t r0 = v / 65535u;
    const uint32_t t0 = v - r0 * 65535u;
    uint32_t r = r0 + ((((t0 * 40503u) & 0xFFFFu) * regions) >> 16);
    if (r >= regions) r -= regions;
    const uint32_t base = r * B;
    uint32_t hb = (((v * 2654435761u) >> 16) * B) >> 16;
    const uint32_t pat = t0 * 0x00010001u;
    for (uint32_t probes = 0; probes < B;) {
        uint32_t* bp = tab32 + (base + hb) * 4;
        const uint4 s = *reinterpret_cast<const uint4*>(bp);
        if (any_zero_half(s.x ^ pat) | any_zero_half(s.y ^ pat) | any_zero_half(s.z ^ pat) | any_zero_half(s.w ^ pat))
            return false;
        int e = -1;
        uint32_t word = 0;
        if (any_zero_half(~s.x)) { e = 0; word = s.x; }
        else if (any_zero_half(~s.y)) { e = 1; word = s.y; }
        else if (any_zero_half(~s.z)) { e = 2; word = s.z; }
        else if (any_zero_half(~s.w)) { e = 3; word = s.w; }
        if (e < 0) {
            hb = hb + 1 == B ? 0 : hb + 1;
            ++probes;
            continue;
        }
        if (!may_insert) return true;
        const uint32_t want = (word & 0xFFFFu) == 0xFFFFu ? ((word & 0xFFFF0000u) | t0) : ((word & 0xFFFFu) | (t0 << 16));
        if (atomicCAS(bp + e, word, want) == word) return true;
        // the word changed under us: look at this bucket again
    }
    failed = true;
    return true;  // no room: the node is evaluated (possibly again); the merge drops duplicates
}

// ---------------------------------------------------------------------------------------------
// Visited set as a cache (the other mode of the same two table formats): an id is looked up and kept
// in its home bucket only; when the bucket has no free slot the id takes the place of another one,
// which is thereby forgotten and may be evaluated again later -- harmless for the list (see
// merge_new_keys), cheaper in LDS.  A lookup never reports an id that was not put in (entries identify
// ids exactly), and an id that is still in its bucket is always found.
// Both return true when v was not in the table; `evicted` is raised when an id was displaced.
// 32-bit entries: four ids per bucket; a slot is claimed by compare-and-swap (two lanes that want the same
// slot: exactly one wins, the other looks again), the victim of a full bucket is chosen by `clock`.
__device__ __forceinline__ bool visited32_cache(uint32_t* tab, int bucket_bits, uint32_t v, uint32_t clock,
                                                bool& evicted) {
    uint32_t* bp = tab + ((v * 2654435761u) >> (32 - bucket_bits)) * 4;
    for (;;) {  // ends: a failed compare-and-swap means another lane's succeeded, and a lane stops at its first success
        const uint4 s = *reinterpret_cast<const uint4*>(bp);
        if (s.x == v || s.y == v || s.z == v || s.w == v) return false;
        int e = s.x == EMPTY_ID ? 0 : (s.y == EMPTY_ID ? 1 : (s.z == EMPTY_ID ? 2 : (s.w == EMPTY_ID ? 3 : -1)));
        const bool full = e < 0;
        if (full) e = (int)(clock & 3u);
        const uint32_t seen = e == 0 ? s.x : (e == 1 ? s.y : (e == 2 ? s.z : s.w));
        if (atomicCAS(bp + e, seen, v) == seen) {
            evicted |= full;
            return true;
        }
    }
}

// 16-bit entries: a bucket (16 bytes) holds seven tags and, in the upper half of its last word, the number of tags
// ever put into it.  A lookup reads the bucket and compares seven halves; an id that is not there takes the next
// position in turn (count mod 7: first the free ones, then the oldest tag), which it learns from one atomic add on the
// counter -- lanes of one expansion that fall into the same bucket get different counts, so there is no retry loop.
// An adjacency row may name a node twice: both lanes then miss, and the one with the higher count gives way before
// anything is written (the loop below runs once per lane that was not the first of this call in its bucket, a handful
// per expansion).
// Called by all lanes of the wave that are active at the call site (it holds wave-level operations).
typedef unsigned short qv_u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t min_halves(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(qv_u16x2, a), __builtin_bit_cast(qv_u16x2, b)));
}
constexpr uint32_t CACHE16_EMPTY_LAST_WORD = 0x0000FFFFu;   // no tag in the seventh place, count 0

__device__ __forceinline__ bool visited16_cache(uint32_t* tab32, uint32_t regions, uint32_t B, uint32_t v, bool active,
                                                int lane, bool& evicted) {
    const uint32_t r0 = v / 65535u;
    const uint32_t t0 = v - r0 * 65535u;
    uint32_t r = r0 + ((((t0 * 40503u) & 0xFFFFu) * regions) >> 16);
    if (r >= regions) r -= regions;
    const uint32_t hb = (((v * 2654435761u) >> 16) * B) >> 16;
    const uint32_t pat = t0 * 0x00010001u;
    uint32_t* bp = tab32 + (r * B + hb) * 4;
    uint4 s = make_uint4(0u, 0u, 0u, 0u);
    if (active) s = *reinterpret_cast<const uint4*>(bp);
    // a half of s equal to the tag shows as a zero half of s ^ pat; the counter's half is kept from ever matching
    const uint32_t x = min_halves(min_halves(s.x ^ pat, s.y ^ pat), min_halves(s.z ^ pat, (s.w ^ pat) | 0xFFFF0000u));
    bool fresh = active && any_zero_half(x) == 0u;
    const uint32_t before = s.w >> 16;   // the bucket's count when this call began (every lane reads before any lane adds)
    uint32_t count = before;
    if (fresh) count = atomicAdd(bp + 3, 0x00010000u) >> 16;
    uint64_t later = __ballot(fresh && count != before);
    while (later) {
        const int j = __ffsll((unsigned long long)later) - 1;
        later &= later - 1;
        const uint32_t vj = (uint32_t)__builtin_amdgcn_readlane((int)v, j);
        const uint32_t cj = (uint32_t)__builtin_amdgcn_readlane((int)count, j);
        const bool twin_before = __any(fresh && v == vj && count < cj);   // same id => same bucket => comparable counts
        if (twin_before && lane == j) fresh = false;                     // (its turn in the bucket stays unused)
    }
    if (fresh) {
        reinterpret_cast<uint16_t*>(bp)[count % 7u] = (uint16_t)t0;
        evicted |= count >= 7u;
    }
    return fresh;
}

template <int P>
struct Pool {
    uint64_t key[P];
    int size;
};

// Merge the candidate keys `mine` (one per lane, KEY_NONE where a lane has none) into the sorted pool.
// With check_dup, a key whose (dist, id) is already in the pool, or is held by a lower lane too, is
// dropped first: that only happens after the visited table stopped taking ids, and then a
// re-evaluated node is either still in the pool (dropped here) or was rejected/evicted before, in
// which case it is above the current worst key -- the worst key never grows once the pool is full --
// and is filtered out by the first test below.
template <int P>
__device__ __forceinline__ void merge_new_keys(Pool<P>& pool, uint64_t mine, int ef, int lane, bool check_dup,
                                               uint64_t* skeys) {
    uint64_t worst = KEY_NONE;  // key of the last slot: KEY_NONE while the pool has room
#pragma unroll
    for (int r = 0; r < P; ++r)
        if (r == ((ef - 1) >> 6)) worst = readlane64(pool.key[r], (ef - 1) & 63);
    uint64_t qual = __ballot(mine < worst);
    if (check_dup && qual) {
        uint64_t scan = qual;
        while (scan) {
            const int j = __ffsll((unsigned long long)scan) - 1;
            scan &= scan - 1;
            const uint64_t nk = readlane64(mine, j);
            bool dup = lane < j && mine == nk;
#pragma unroll
            for (int r = 0; r < P; ++r) dup |= (pool.key[r] >> 1) == (nk >> 1);
            if (__any(dup)) qual &= ~(1ull << j);
        }
    }
    if (!qual) return;
    const bool is_new = (qual >> lane) & 1ull;

    uint32_t up[P];       // pool entries: number of new keys below them
    uint32_t my_pos = 0;  // new keys: number of pool keys and of other new keys below them
#pragma unroll
    for (int r = 0; r < P; ++r) up[r] = 0;
    uint64_t scan = qual;
    while (scan) {
        const int j = __ffsll((unsigned long long)scan) - 1;
        scan &= scan - 1;
        const uint64_t nk = readlane64(mine, j);
        uint32_t below = 0;
#pragma unroll
        for (int r = 0; r < P; ++r) {
            const bool lt = pool.key[r] < nk;
            below += (uint32_t)__popcll(__ballot(lt));
            up[r] += lt ? 0u : 1u;
        }
        if (lane == j) my_pos += below;
        my_pos += (is_new && nk < mine) ? 1u : 0u;
    }
    const int new_size = min(ef, pool.size + (int)__popcll(qual));
    wave_sync();
#pragma unroll
    for (int r = 0; r < P; ++r) {
        const uint32_t np = (uint32_t)(r * 64 + lane) + up[r];
        if (pool.key[r] != KEY_NONE && np < (uint32_t)ef) skeys[np] = pool.key[r];
    }
    if (is_new && my_pos < (uint32_t)ef) skeys[my_pos] = mine;
    wave_sync();
#pragma unroll
    for (int r = 0; r < P; ++r) {
        const int e = r * 64 + lane;
        pool.key[r] = e < new_size ? skeys[e] : KEY_NONE;
    }
    pool.size = new_size;
}

// The same merge for pools of eight and more registers per lane, where a loop over the new keys that
// touches every pool register is the dominant cost of an expansion.  skeys[0..pool.size) still holds
// the pool as the previous merge left it (sorted; only `expanded` bits may be stale, and they are
// ignored here), so every lane finds the rank of its own key among the pool keys, and whether the
// pool already holds it, by a binary search in LDS, all lanes at once.  What is left for the loop over
// the new keys is wave-uniform data: their pool ranks (a pool entry e moves up by the number of new
// keys whose rank is <= e) and their order among themselves.
template <int P>
__device__ __forceinline__ void merge_new_keys_wide(Pool<P>& pool, uint64_t mine, int ef, int lane, bool check_dup,
                                                    uint64_t* skeys) {
    uint64_t worst = KEY_NONE;
#pragma unroll
    for (int r = 0; r < P; ++r)
        if (r == ((ef - 1) >> 6)) worst = readlane64(pool.key[r], (ef - 1) & 63);
    bool cand = mine < worst;
    uint64_t qual = __ballot(cand);
    if (!qual) return;

    const int n = pool.size;
    const uint64_t k1 = mine >> 1;
    uint32_t rank = 0;  // pool keys whose (dist, id) is below mine
    if (cand) {
        for (int step = n > 0 ? 1 << (31 - __clz(n)) : 0; step > 0; step >>= 1) {
            const uint32_t t = rank + (uint32_t)step;
            if (t <= (uint32_t)n && (skeys[t - 1] >> 1) < k1) rank = t;
        }
        if (check_dup && rank < (uint32_t)n && (skeys[rank] >> 1) == k1) cand = false;  // the pool holds it already
    }
    if (check_dup) {
        qual = __ballot(cand);
        if (!qual) return;
    }

    uint32_t up[P];
#pragma unroll
    for (int r = 0; r < P; ++r) up[r] = 0;
    uint32_t my_pos = rank;
    uint64_t twins = 0;   // lanes whose key a lower lane holds as well
    uint64_t scan = qual;
    while (scan) {
        const int j = __ffsll((unsigned long long)scan) - 1;
        scan &= scan - 1;
        if ((twins >> j) & 1ull) {
            qual &= ~(1ull << j);
            continue;
        }
        const uint64_t nk = readlane64(mine, j);
        const uint32_t rj = (uint32_t)__builtin_amdgcn_readlane((int)rank, j);
        if (check_dup) twins |= __ballot(cand && lane > j && mine == nk);
#pragma unroll
        for (int r = 0; r < P; ++r) up[r] += (uint32_t)(r * 64 + lane) >= rj ? 1u : 0u;
        my_pos += (cand && nk < mine) ? 1u : 0u;
    }
    const bool is_new = (qual >> lane) & 1ull;
    const int new_size = min(ef, n + (int)__popcll(qual));
    wave_sync();
#pragma unroll
    for (int r = 0; r < P; ++r) {
        const uint32_t np = (uint32_t)(r * 64 + lane) + up[r];
        if (pool.key[r] != KEY_NONE && np < (uint32_t)ef) skeys[np] = pool.key[r];
    }
    if (is_new && my_pos < (uint32_t)ef) skeys[my_pos] = mine;
    wave_sync();
#pragma unroll
    for (int r = 0; r < P; ++r) {
        const int e = r * 64 + lane;
        pool.key[r] = e < new_size ? skeys[e] : KEY_NONE;
    }
    pool.size = new_size;
}

// ---------------------------------------------------------------------------------------------
// Stage 2 (paper Sec. 3.3) by the wave that just finished Stage 1 of a query: exact cosine between the float32
// query and every member of the final list, best k by (score descending, id ascending).  Four candidates at a
// time: their rows are streamed with coalesced 16-byte loads (all loads of the four rows in flight together when the
// width is known at compile time), dot product and squared norm are accumulated in double per lane, and the eight
// per-lane sums are reduced together -- each exchange step halves what a lane still carries, so the wave-wide
// reduction of eight values costs 20 lane exchanges instead of 96.  Scores and ids go to LDS (the merge area, which
// is free by now), ranks come from counting.
__device__ __forceinline__ double lane_xor_f64(double v, int mask) { return __shfl_xor(v, mask); }

template <int NW_T, int P>
__device__ __forceinline__ void rerank_own_list(const SearchParams& p, int64_t q, const Pool<P>& pool, int lane, uint64_t* skeys) {
    const int d = p.rr_d, nc = pool.size, k = p.rr_k;
    const float* qf = p.rr_queries + q * (int64_t)d;
    float* s_score = reinterpret_cast<float*>(skeys);              // [64 * P]
    uint32_t* s_id = reinterpret_cast<uint32_t*>(s_score + 64 * P);  // [64 * P]
    const bool vec4 = (d & 3) == 0;
    const int d4 = d >> 2;
    constexpr int IT = NW_T > 0 ? (NW_T + 3) / 4 : 2;   // float4 per lane and row when the width is known
    constexpr int CH = IT < 4 ? IT : 4;

    double qq = 0.0;
    if (vec4) {
        const float4* q4 = reinterpret_cast<const float4*>(qf);
        for (int i = lane; i < d4; i += 64) {
            const float4 a = q4[i];
            qq += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
        }
    } else {
        for (int i = lane; i < d; i += 64) qq += (double)qf[i] * (double)qf[i];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) qq += lane_xor_f64(qq, off);

    wave_sync();  // the merge area is read as keys no more
    for (int c0 = 0; c0 < nc; c0 += 4) {
        uint32_t id[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = min(c0 + j, nc - 1);   // beyond the list: the last member again, result dropped
            uint32_t v = 0;
#pragma unroll
            for (int r = 0; r < P; ++r)
                if (r == (c >> 6)) v = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(pool.key[r] >> 1), c & 63);
            id[j] = v;
        }
        double acc[8];   // dot0, xx0, dot1, xx1, dot2, xx2, dot3, xx3
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0;
        if (vec4) {
            // CH float4 per lane and row at a time: all loads of a chunk (four rows and the query) before its arithmetic
            const float4* q4 = reinterpret_cast<const float4*>(qf);
            for (int base = 0; base < d4; base += 64 * CH) {
                float4 xv[4][CH], qv4[CH];
#pragma unroll
                for (int it = 0; it < CH; ++it) {
                    const int i = min(base + it * 64 + lane, d4 - 1);   // clamped: masked below
                    qv4[it] = q4[i];
#pragma unroll
                    for (int j = 0; j < 4; ++j) xv[j][it] = reinterpret_cast<const float4*>(p.rr_vecs + (int64_t)id[j] * d)[i];
                }
#pragma unroll
                for (int it = 0; it < CH; ++it) {
                    if (base + it * 64 + lane < d4) {
                        const float4 b = qv4[it];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const float4 a = xv[j][it];
                            acc[2 * j] += (double)a.x * b.x + (double)a.y * b.y + (double)a.z * b.z + (double)a.w * b.w;
                            acc[2 * j + 1] += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
                        }
                    }
                }
            }
        } else {
            for (int i = lane; i < d; i += 64) {
                const double b = qf[i];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const double a = p.rr_vecs[(int64_t)id[j] * d + i];
                    acc[2 * j] += a * b;
                    acc[2 * j + 1] += a * a;
                }
            }
        }
        // eight sums over 64 lanes: halves of the wave keep candidates {0,1} / {2,3}, then quarters one candidate each,
        // then eighths either its dot product or its squared norm; three plain steps finish inside groups of eight
        double h4[4], h2[2], v;
        {
            const bool up = lane & 32;
#pragma unroll
            for (int j = 0; j < 4; ++j) h4[j] = (up ? acc[4 + j] : acc[j]) + lane_xor_f64(up ? acc[j] : acc[4 + j], 32);
        }
        {
            const bool up = lane & 16;
#pragma unroll
            for (int j = 0; j < 2; ++j) h2[j] = (up ? h4[2 + j] : h4[j]) + lane_xor_f64(up ? h4[j] : h4[2 + j], 16);
        }
        {
            const bool up = lane & 8;
            v = (up ? h2[1] : h2[0]) + lane_xor_f64(up ? h2[0] : h2[1], 8);
        }
        v += lane_xor_f64(v, 4);
        v += lane_xor_f64(v, 2);
        v += lane_xor_f64(v, 1);
        const double other = lane_xor_f64(v, 8);   // lanes 0, 16, 32, 48: v = dot, other = squared norm of candidate lane / 16
        if ((lane & 15) == 0) {
            const int j = lane >> 4;
            if (c0 + j < nc) {
                float sc = 0.0f;
                if (qq != 0.0 && other != 0.0) sc = (float)(v / (sqrt(qq) * sqrt(other)));
                if (sc != sc) sc = -__builtin_inff();   // a stored vector with Inf or NaN in it ranks last
                s_score[c0 + j] = sc;
                s_id[c0 + j] = j == 0 ? id[0] : (j == 1 ? id[1] : (j == 2 ? id[2] : id[3]));
            }
        }
    }
    wave_sync();
    // rank by counting: position of candidate t = number of candidates that come before it
#pragma unroll
    for (int r = 0; r < P; ++r) {
        const int t = r * 64 + lane;
        if (t < nc) {
            const float st = s_score[t];
            const uint32_t it = s_id[t];
            int rank = 0;
            for (int j = 0; j < nc; ++j) {
                const float sj = s_score[j];
                const uint32_t ij = s_id[j];
                rank += (sj > st || (sj == st && ij < it)) ? 1 : 0;
            }
            if (rank < k) {
                p.rr_ids[q * (int64_t)k + rank] = it;
                p.rr_scores[q * (int64_t)k + rank] = st;
            }
        }
    }
    for (int r = nc + lane; r < k; r += 64) {
        p.rr_ids[q * (int64_t)k + r] = EMPTY_ID;
        p.rr_scores[q * (int64_t)k + r] = -__builtin_inff();
    }
}

// Stage 2 by another wave of the same launch (SearchParams::rr_ticket).  The two waves may sit on different compute
// dies, whose L2 caches do not see each other's ordinary stores until a kernel ends; flushing and invalidating those
// caches per query (what a release / acquire fence at device scope does) costs more than the whole stage.  So what
// has to travel -- the list's ids, its length, the flag -- is written and read with device-coherent accesses
// (relaxed atomics at device scope: they go to the memory side of the L2s), ordered by waiting for the stores to
// be acknowledged before the flag is written and for the flag to arrive before the list is read.
__device__ __forceinline__ void coherent_store(uint32_t* at, uint32_t v) {
    __hip_atomic_store(at, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t coherent_load(const uint32_t* at) {
    return __hip_atomic_load(at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// the searching wave, after its coherent stores of the list: raise the query's flag
__device__ __forceinline__ void publish_list(const SearchParams& p, int64_t q, int lane) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // every lane's stores of this wave are acknowledged
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) coherent_store(p.rr_done + q, 1u);
}

// The scoring wave: waits for the flag (the search it waits for is running, see SearchParams), reads the list from
// memory into the register layout of a pool and scores it as rerank_own_list does.
template <int NW_T, int P>
__device__ __forceinline__ void score_finished_list(const SearchParams& p, int64_t q, int lane, uint64_t* lds) {
    uint32_t ready = 0;
    if (lane == 0) {
        for (uint32_t polls = 0;; ++polls) {
            ready = coherent_load(p.rr_done + q);
            if (ready || polls >= p.rr_spin_limit) break;
            __builtin_amdgcn_s_sleep(64);
        }
    }
    ready = (uint32_t)__builtin_amdgcn_readfirstlane((int)ready);   // (waits for the flag's load)
    asm volatile("" ::: "memory");
    Pool<P> pool;
    pool.size = ready ? (int)coherent_load(p.n_cand + q) : 0;
#pragma unroll
    for (int r = 0; r < P; ++r) {
        const int e = r * 64 + lane;
        pool.key[r] = e < pool.size ? (uint64_t)coherent_load(p.cand_ids + q * (int64_t)p.ef + e) << 1 : KEY_NONE;
    }
    // gave up (never seen in a working launch): an empty, flagged result
    if (!ready && lane == 0 && p.status) p.status[q] = QV_STATUS_TIMEOUT_BIT;
    rerank_own_list<NW_T, P>(p, q, pool, lane, lds);
}

// lanes `sub` of a group that ends up with the sum of pass b after the reduce-scatter below (and its inverse)
template <int G>
__device__ __forceinline__ constexpr int lane_of_pass(int b) { return G == 4 ? ((b >> 1) | ((b & 1) << 1)) : b; }

template <int ENC, int NW_T, int G, int P, bool NARROW, bool SPLIT>
__global__ __launch_bounds__(64) void beam_search_kernel(SearchParams p) {
    extern __shared__ __align__(16) uint32_t smem[];
    const int lane = threadIdx.x;
    int64_t slot = blockIdx.x;
    if constexpr (P <= 2) {
        if (p.rr_ticket) {   // roles by ticket, in the order in which workgroups start (see SearchParams)
            uint32_t t = 0;
            if (lane == 0) t = atomicAdd(p.rr_ticket, 1u);
            slot = (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)t);
            if (slot >= p.nq) {
                score_finished_list<NW_T, P>(p, p.order ? (int64_t)p.order[slot - p.nq] : slot - p.nq, lane,
                                             reinterpret_cast<uint64_t*>(smem));
                return;
            }
        }
    }
    const int64_t q = p.order ? (int64_t)p.order[slot] : slot;
    const int NW = NW_T > 0 ? NW_T : p.nw;
    if (p.qstatus && (p.qstatus[q] & QV_STATUS_NONFINITE_BIT)) {   // wave-uniform
        // a query with Inf or NaN in it has no code to search with: empty list, no results, the flag in its status
        for (int e = lane; e < p.ef; e += 64) {
            if (p.cand_ids) p.cand_ids[q * (int64_t)p.ef + e] = EMPTY_ID;
            if (p.cand_dist) p.cand_dist[q * (int64_t)p.ef + e] = EMPTY_ID;
        }
        if (p.visit_order)
            for (int64_t i = lane; i < p.visit_cap; i += 64) p.visit_order[q * p.visit_cap + i] = EMPTY_ID;
        if (p.rr_vecs && !p.rr_ticket)
            for (int r = lane; r < p.rr_k; r += 64) {
                p.rr_ids[q * (int64_t)p.rr_k + r] = EMPTY_ID;
                p.rr_scores[q * (int64_t)p.rr_k + r] = -__builtin_inff();
            }
        if (lane == 0) {
            if (p.n_cand) {
                if (p.rr_ticket) coherent_store(p.n_cand + q, 0u);
                else p.n_cand[q] = 0;
            }
            if (p.n_expanded) p.n_expanded[q] = 0;
            if (p.n_evals) p.n_evals[q] = 0;
            if (p.status) p.status[q] = QV_STATUS_NONFINITE_BIT;
        }
        if (p.rr_ticket) publish_list(p, q, lane);   // the scoring wave pads the result of an empty list
        return;
    }
    const uint32_t cap = p.vis_slots;   // slots (32-bit each, or 16-bit when NARROW)
    const uint32_t vis_regions = p.vis_regions, vis_B = p.vis_region_buckets;
    const uint32_t vis_used = NARROW ? vis_regions * vis_B * 8 : cap;
    const uint32_t vis_limit = vis_used - (vis_used >> 2) - 64;  // stop inserting at 3/4 full
    const uint32_t tab_words = NARROW ? cap >> 1 : cap;
    const int bucket_bits = p.vis_bucket_bits;
    const uint32_t bucket_mask = (1u << bucket_bits) - 1;
    const bool cache_mode = p.vis_cache != 0;
    uint32_t* tab = smem;
    uint32_t* list = tab + tab_words;  // [64] compacted new neighbour ids
    uint32_t* dlist = list + 64;       // [64] their distances (generic gather path)
    uint64_t* skeys = reinterpret_cast<uint64_t*>(dlist + 64);  // [64*P + 64] merge scatter area
    uint64_t* qlds = skeys + 64 * P + 64;                      // [3*NW] query words (generic path)

    const uint32_t last_word = (NARROW && cache_mode) ? CACHE16_EMPTY_LAST_WORD : EMPTY_ID;
    for (uint32_t i = lane * 4; i < tab_words; i += 256)
        *reinterpret_cast<uint4*>(tab + i) = make_uint4(EMPTY_ID, EMPTY_ID, EMPTY_ID, last_word);

    constexpr int RPP = 64 / G;  // neighbour rows per pass
    constexpr int KW = NW_T > 0 ? (NW_T + G - 1) / G : 1;
    // passes whose loads are in flight together: all G of them unless that needs > 48 x 64-bit registers
    constexpr int BATCH = (2 * KW * G <= 48) ? G : (48 / (2 * KW) > 0 ? 48 / (2 * KW) : 1);
    // with all passes in one batch and groups inside a quad, the lane sums are combined by a
    // reduce-scatter over data-parallel primitives and never go through LDS
    constexpr bool QUAD_REDUCE = NW_T > 0 && BATCH == G && (G == 1 || G == 2 || G == 4);
    // word assignment inside a group: interleaved (lane s takes words s, s+G, ...) or, when every lane gets
    // an even number of words, blocked (lane s takes words s*KW .. s*KW+KW-1) so that two words travel
    // in one 16-byte load
    constexpr bool BLOCKED = QUAD_REDUCE && NW_T % (2 * G) == 0;
    const int sub = lane % G, grp = lane / G;
    constexpr int PLANES = ENC == ENC_SIGN1 ? 1 : 2;
    const int RW = PLANES * NW;  // 64-bit words per code row
    const uint64_t* qsrc = p.qcodes + q * (int64_t)RW;
    uint64_t qp[KW], qs[KW], q3[KW];
    if constexpr (NW_T > 0) {
#pragma unroll
        for (int i = 0; i < KW; ++i) {
            int w = BLOCKED ? sub * KW + i : sub + i * G;
            const uint64_t a = w < NW_T ? qsrc[w] : 0ull;
            const uint64_t b = (PLANES == 2 && w < NW_T) ? qsrc[NW_T + w] : 0ull;
            code_query_words<ENC>(a, b, qp[i], qs[i], q3[i]);
        }
    } else {
        for (int w = lane; w < NW; w += 64) {
            uint64_t q0, q1, q2;
            code_query_words<ENC>(qsrc[w], PLANES == 2 ? qsrc[NW + w] : 0ull, q0, q1, q2);
            qlds[w] = q0; qlds[NW + w] = q1; qlds[2 * NW + w] = q2;
        }
        qp[0] = qs[0] = q3[0] = 0;
    }

    Pool<P> pool;
#pragma unroll
    for (int r = 0; r < P; ++r) pool.key[r] = KEY_NONE;
    pool.size = 0;
    const int ef = p.ef;
    uint32_t n_vis = 0, n_exp = 0, n_eval = 0, status = 0;
    bool vis_full = false;
    uint32_t* order = p.visit_order ? p.visit_order + q * p.visit_cap : nullptr;

    wave_sync();

    // distances of list[0..m) -> merge into the pool
    auto process_list = [&](int m) {
        wave_sync();  // list[] written by other lanes
        uint64_t mine = KEY_NONE;
        if constexpr (SPLIT) {
            // Two steps.  First the sign plane and the K1 magnitude words that share its lines: with the unknown
            // magnitude words taken as zero, Table 1's sum is a lower bound of the distance (a differing sign then
            // counts (1 + strong_q) instead of (1 + strong_q)(1 + strong_v)).  A neighbour whose bound is not below
            // the list's worst key cannot enter the list whatever the rest of its code says, so the remaining
            // magnitude words are read only for the others, and the bound is completed to the exact distance:
            // per word the missing part is pc(X and s_v) + pc(X and s_v and s_q).
            static_assert(QUAD_REDUCE && BLOCKED && ENC == ENC_SM, "split rows: two or four lanes per row, blocked words");
            constexpr int K1 = split_k1(NW_T), S1 = split_stride1(NW_T), S2 = split_stride2(NW_T);
            uint64_t worst = KEY_NONE;  // key of the last slot: KEY_NONE while the pool has room
#pragma unroll
            for (int r = 0; r < P; ++r)
                if (r == ((ef - 1) >> 6)) worst = readlane64(pool.key[r], (ef - 1) & 63);
            uint64_t xv[G][KW], sv[G][KW];
#pragma unroll
            for (int b = 0; b < G; ++b) {
                if (b * RPP < m) {  // wave-uniform
                    const int ri = min(b * RPP + grp, m - 1);
                    const uint64_t* row = p.codes1 + (int64_t)list[ri] * S1;
                    const uint4* r4 = reinterpret_cast<const uint4*>(row + sub * KW);
                    const uint4* m4 = reinterpret_cast<const uint4*>(row + NW_T + sub * KW);
#pragma unroll
                    for (int i = 0; i < KW / 2; ++i) {
                        const uint4 a = r4[i];
                        xv[b][2 * i] = ((uint64_t)a.y << 32) | a.x;
                        xv[b][2 * i + 1] = ((uint64_t)a.w << 32) | a.z;
                        uint4 c = make_uint4(0u, 0u, 0u, 0u);
                        if (sub * KW + 2 * i < K1) c = m4[i];   // K1 is even: a pair of words is in one array or the other
                        sv[b][2 * i] = ((uint64_t)c.y << 32) | c.x;
                        sv[b][2 * i + 1] = ((uint64_t)c.w << 32) | c.z;
                    }
                }
            }
            uint32_t part[G];
#pragma unroll
            for (int b = 0; b < G; ++b) {
                uint32_t c1 = 0, c2 = 0, c3 = 0;
                if (b * RPP < m) {  // wave-uniform
#pragma unroll
                    for (int i = 0; i < KW; ++i) {
                        sm_accumulate(xv[b][i], sv[b][i], qp[i], qs[i], c1, c2, c3);
                        xv[b][i] ^= qp[i];   // the differing signs, kept for the second step
                    }
                }
                part[b] = c1 + c2 + 2u * c3;
            }
            auto reduce_scatter = [&](const uint32_t* v, int& my_b) -> uint32_t {
                if constexpr (G == 2) {
                    const bool hi = sub & 1;
                    my_b = hi ? 1 : 0;
                    return (hi ? v[1] : v[0]) + quad_xor1(hi ? v[0] : v[1]);
                } else {
                    const bool o1 = sub & 1, o2 = sub & 2;
                    const uint32_t k0 = (o1 ? v[2] : v[0]) + quad_xor1(o1 ? v[0] : v[2]);
                    const uint32_t k1 = (o1 ? v[3] : v[1]) + quad_xor1(o1 ? v[1] : v[3]);
                    my_b = (o1 ? 2 : 0) + (o2 ? 1 : 0);
                    return (o2 ? k1 : k0) + quad_xor2(o2 ? k0 : k1);
                }
            };
            int my_b;
            uint32_t dist = reduce_scatter(part, my_b);
            const int my_ri = my_b * RPP + grp;
            const uint32_t my_id = my_ri < m ? list[my_ri] : 0u;
            const uint64_t bound_key = ((uint64_t)dist << 33) | ((uint64_t)my_id << 1);
            const uint64_t open = __ballot(my_ri < m && bound_key < worst);   // bit grp*G + lane_of_pass(b): row b*RPP + grp goes on
            if (open) {
                uint32_t rest[G];
#pragma unroll
                for (int b = 0; b < G; ++b) {
                    rest[b] = 0;
                    const bool go = (open >> (grp * G + lane_of_pass<G>(b))) & 1ull;
                    if (__any(go)) {
                        uint64_t s2[KW];
                        const uint64_t* row = p.codes2 + (int64_t)list[min(b * RPP + grp, m - 1)] * S2;
#pragma unroll
                        for (int i = 0; i < KW / 2; ++i) {
                            uint4 c = make_uint4(0u, 0u, 0u, 0u);
                            const int w = sub * KW + 2 * i;
                            if (go && w >= K1) c = *reinterpret_cast<const uint4*>(row + (w - K1));
                            s2[2 * i] = ((uint64_t)c.y << 32) | c.x;
                            s2[2 * i + 1] = ((uint64_t)c.w << 32) | c.z;
                        }
                        uint32_t e = 0;
#pragma unroll
                        for (int i = 0; i < KW; ++i) {
                            const uint64_t t = xv[b][i] & s2[i];
                            e += __popcll(t) + __popcll(t & qs[i]);
                        }
                        rest[b] = e;
                    }
                }
                int same_b;
                dist += reduce_scatter(rest, same_b);
            }
            if (my_ri < m) mine = ((uint64_t)dist << 33) | ((uint64_t)my_id << 1);
        } else if constexpr (QUAD_REDUCE) {
            // pass b handles row b*RPP + grp; all loads first, then the arithmetic.  Lanes beyond the list load
            // the list's last row instead of being masked off (the line is in flight anyway, no branch, no
            // zero fill); what they compute is never used.
            uint64_t pv[G][KW], sv[G][KW];
#pragma unroll
            for (int b = 0; b < G; ++b) {
                if (b * RPP < m) {  // wave-uniform
                    const int ri = min(b * RPP + grp, m - 1);
                    const uint64_t* row = p.codes + (uint64_t)list[ri] * (uint32_t)p.row_stride;
                    if constexpr (BLOCKED) {
                        const uint4* r4 = reinterpret_cast<const uint4*>(row + sub * KW);
                        const uint4* m4 = reinterpret_cast<const uint4*>(row + NW_T + sub * KW);
#pragma unroll
                        for (int i = 0; i < KW / 2; ++i) {
                            const uint4 a = r4[i];
                            pv[b][2 * i] = ((uint64_t)a.y << 32) | a.x;
                            pv[b][2 * i + 1] = ((uint64_t)a.w << 32) | a.z;
                            if constexpr (PLANES == 2) {
                                const uint4 c = m4[i];
                                sv[b][2 * i] = ((uint64_t)c.y << 32) | c.x;
                                sv[b][2 * i + 1] = ((uint64_t)c.w << 32) | c.z;
                            } else {
                                sv[b][2 * i] = sv[b][2 * i + 1] = 0ull;
                            }
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < KW; ++i) {
                            int w = sub + i * G;
                            pv[b][i] = w < NW_T ? row[w] : 0ull;
                            sv[b][i] = (PLANES == 2 && w < NW_T) ? row[NW_T + w] : 0ull;
                        }
                    }
                }
            }
            uint32_t part[G];
#pragma unroll
            for (int b = 0; b < G; ++b) {
                uint32_t c1 = 0, c2 = 0, c3 = 0;
                if (b * RPP < m) {  // wave-uniform
#pragma unroll
                    for (int i = 0; i < KW; ++i) {
                        code_accumulate<ENC>(pv[b][i], sv[b][i], qp[i], qs[i], q3[i], c1, c2, c3);
                    }
                }
                part[b] = code_distance_from_counts<ENC>(c1, c2, c3);
            }
            // reduce-scatter: afterwards lane `sub` holds the full sum of pass my_b
            uint32_t dist;
            int my_b;
            if constexpr (G == 1) {
                dist = part[0];
                my_b = 0;
            } else if constexpr (G == 2) {
                const bool hi = sub & 1;
                dist = (hi ? part[1] : part[0]) + quad_xor1(hi ? part[0] : part[1]);
                my_b = hi ? 1 : 0;
            } else {
                const bool o1 = sub & 1, o2 = sub & 2;
                uint32_t k0 = (o1 ? part[2] : part[0]) + quad_xor1(o1 ? part[0] : part[2]);
                uint32_t k1 = (o1 ? part[3] : part[1]) + quad_xor1(o1 ? part[1] : part[3]);
                dist = (o2 ? k1 : k0) + quad_xor2(o2 ? k0 : k1);
                my_b = (o1 ? 2 : 0) + (o2 ? 1 : 0);
            }
            const int my_ri = my_b * RPP + grp;
            if (my_ri < m) mine = ((uint64_t)dist << 33) | ((uint64_t)list[my_ri] << 1);
        } else {
            if constexpr (NW_T > 0) {
                for (int base = 0; base < m; base += RPP * BATCH) {
                    uint64_t pv[BATCH][KW], sv[BATCH][KW];
#pragma unroll
                    for (int b = 0; b < BATCH; ++b) {
                        int ri = base + b * RPP + grp;
                        if (ri < m) {
                            const uint64_t* row = p.codes + (uint64_t)list[ri] * (uint32_t)p.row_stride;
#pragma unroll
                            for (int i = 0; i < KW; ++i) {
                                int w = sub + i * G;
                                pv[b][i] = w < NW_T ? row[w] : 0ull;
                                sv[b][i] = (PLANES == 2 && w < NW_T) ? row[NW_T + w] : 0ull;
                            }
                        } else {
#pragma unroll
                            for (int i = 0; i < KW; ++i) pv[b][i] = sv[b][i] = 0ull;
                        }
                    }
#pragma unroll
                    for (int b = 0; b < BATCH; ++b) {
                        int ri = base + b * RPP + grp;
                        if (base + b * RPP < m) {  // wave-uniform
                            uint32_t c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
                            for (int i = 0; i < KW; ++i) {
                                code_accumulate<ENC>(pv[b][i], sv[b][i], qp[i], qs[i], q3[i], c1, c2, c3);
                            }
                            uint32_t dist = code_distance_from_counts<ENC>(c1, c2, c3);
#pragma unroll
                            for (int off = G >> 1; off >= 1; off >>= 1) dist += __shfl_xor((int)dist, off);
                            if (sub == 0 && ri < m) dlist[ri] = dist;
                        }
                    }
                }
            } else {
                for (int base = 0; base < m; base += RPP) {
                    int ri = base + grp;
                    uint32_t c1 = 0, c2 = 0, c3 = 0;
                    if (ri < m) {
                        const uint64_t* row = p.codes + (uint64_t)list[ri] * (uint32_t)p.row_stride;
                        for (int w = sub; w < NW; w += G) {
                            code_accumulate<ENC>(row[w], PLANES == 2 ? row[NW + w] : 0ull, qlds[w], qlds[NW + w],
                                                 qlds[2 * NW + w], c1, c2, c3);
                        }
                    }
                    uint32_t dist = code_distance_from_counts<ENC>(c1, c2, c3);
#pragma unroll
                    for (int off = G >> 1; off >= 1; off >>= 1) dist += __shfl_xor((int)dist, off);
                    if (sub == 0 && ri < m) dlist[ri] = dist;
                }
            }
            wave_sync();
            if (lane < m) mine = ((uint64_t)dlist[lane] << 33) | ((uint64_t)list[lane] << 1);
        }
        n_eval += (uint32_t)m;
        if constexpr (P >= 8) merge_new_keys_wide<P>(pool, mine, ef, lane, vis_full, skeys);
        else merge_new_keys<P>(pool, mine, ef, lane, vis_full, skeys);
    };

    // the entry node
    if (lane == 0) {
        list[0] = p.entry;
        bool ignore = false;
        if (cache_mode) {
            if constexpr (NARROW) visited16_cache(tab, vis_regions, vis_B, p.entry, true, lane, ignore);
            else visited32_cache(tab, bucket_bits, p.entry, 0u, ignore);
        } else {
            if constexpr (NARROW) visited16_test_and_set(tab, vis_regions, vis_B, p.entry, true, ignore);
            else visited32_test_and_set(tab, bucket_mask, bucket_bits, p.entry, true);
        }
    }
    n_vis = 1;
    process_list(1);

    // adjacency row (first 64 slots) of the runner-up, loaded ahead of time: when the next expansion
    // picks that node -- the usual case once the pool has settled -- its row is already here
    uint32_t pre_uid = EMPTY_ID, pre_v = EMPTY_ID;
    for (;;) {
        // best unexpanded entry, and the one after it
        uint32_t uid = EMPTY_ID, uid2 = EMPTY_ID;
        int n_found = 0;
#pragma unroll
        for (int r = 0; r < P; ++r) {
            if (n_found < 2) {
                uint64_t open = __ballot(pool.key[r] != KEY_NONE && !(pool.key[r] & 1ull));
                if (open && n_found == 0) {
                    int l = __ffsll((unsigned long long)open) - 1;
                    uid = (uint32_t)(readlane64(pool.key[r], l) >> 1);
                    if (lane == l) pool.key[r] |= 1ull;
                    open &= open - 1;
                    n_found = 1;
                }
                if (open && n_found == 1) {
                    int l = __ffsll((unsigned long long)open) - 1;
                    uid2 = (uint32_t)(readlane64(pool.key[r], l) >> 1);
                    n_found = 2;
                }
            }
        }
        if (n_found == 0) break;
        if (order && lane == 0 && (int64_t)n_exp < p.visit_cap) order[n_exp] = uid;
        n_exp++;
        const bool have_row = uid == pre_uid;
        const uint32_t first_v = pre_v;
        if (uid2 != EMPTY_ID && uid2 != pre_uid) {
            pre_v = lane < p.R ? p.adj[(int64_t)uid2 * p.R + lane] : EMPTY_ID;
            pre_uid = uid2;
        } else if (uid2 == EMPTY_ID) {
            pre_uid = EMPTY_ID;
        }

        const uint32_t* arow = p.adj + (int64_t)uid * p.R;
        for (int c = 0; c < p.R; c += 64) {
            uint32_t v;
            if (c == 0 && have_row) v = first_v;
            else v = (c + lane < p.R) ? arow[c + lane] : EMPTY_ID;
            bool valid = v != EMPTY_ID;
            if (valid && (int64_t)v >= p.n) { valid = false; status |= QV_STATUS_BAD_EDGE_BIT; }
            bool fresh = false;
            if (cache_mode) {
                bool evicted = false;
                if constexpr (NARROW) {
                    fresh = visited16_cache(tab, vis_regions, vis_B, valid ? v : 0u, valid, lane, evicted);
                } else {
                    if (valid) fresh = visited32_cache(tab, bucket_bits, v, n_exp + (uint32_t)lane, evicted);
                }
                if (!vis_full && __any(evicted)) {  // from now on a node may come back: merges check for duplicates
                    vis_full = true;
                    status |= QV_STATUS_VISITED_FULL_BIT;
                }
            } else if constexpr (NARROW) {
                if (!vis_full && n_vis + (uint32_t)__popcll(__ballot(valid)) > vis_limit) {
                    vis_full = true;
                    status |= QV_STATUS_VISITED_FULL_BIT;
                }
                // (with a full table two lanes holding the same id both count as new here; the
                // duplicate check at merge time drops the second one)
                bool failed = false;
                if (valid) fresh = visited16_test_and_set(tab, vis_regions, vis_B, v, !vis_full, failed);
                if (__any(failed)) {  // one part of the table is full: stop inserting altogether
                    vis_full = true;
                    status |= QV_STATUS_VISITED_FULL_BIT;
                }
            } else {
                if (!vis_full && n_vis + (uint32_t)__popcll(__ballot(valid)) > vis_limit) {
                    vis_full = true;
                    status |= QV_STATUS_VISITED_FULL_BIT;
                }
                fresh = valid && visited32_test_and_set(tab, bucket_mask, bucket_bits, v, !vis_full);
            }
            uint64_t fm = __ballot(fresh);
            int m = __popcll(fm);
            if (m == 0) continue;
            n_vis += (uint32_t)m;
            wave_sync();  // previous readers of list[] are done
            if (fresh) list[__popcll(fm & ((1ull << lane) - 1ull))] = v;
            process_list(m);
        }
    }

    // results: sorted list, counters
    if (p.cand_ids) {
        uint32_t* cid = p.cand_ids + q * (int64_t)ef;
        uint32_t* cds = p.cand_dist + q * (int64_t)ef;
#pragma unroll
        for (int r = 0; r < P; ++r) {
            int e = r * 64 + lane;
            if (e < ef) {
                bool has = pool.key[r] != KEY_NONE;
                const uint32_t id = has ? (uint32_t)(pool.key[r] >> 1) : EMPTY_ID;
                if (P <= 2 && p.rr_ticket) coherent_store(cid + e, id);   // read by a wave that may sit on another die
                else cid[e] = id;
                cds[e] = has ? (uint32_t)(pool.key[r] >> 33) : EMPTY_ID;
            }
        }
    }
    status = (uint32_t)__builtin_amdgcn_readfirstlane((int)status) |
             (__any(status & QV_STATUS_BAD_EDGE_BIT) ? QV_STATUS_BAD_EDGE_BIT : 0u);
    if constexpr (P <= 2) {
        if (p.rr_vecs && !p.rr_ticket) rerank_own_list<NW_T, P>(p, q, pool, lane, skeys);
    }
    if (lane == 0) {
        if (p.n_cand) {
            if (P <= 2 && p.rr_ticket) coherent_store(p.n_cand + q, (uint32_t)pool.size);
            else p.n_cand[q] = (uint32_t)pool.size;
        }
        if (p.n_expanded) p.n_expanded[q] = n_exp;
        if (p.n_evals) p.n_evals[q] = n_eval;
        if (p.status) p.status[q] = status;
        if (order)
            for (int64_t i = n_exp; i < p.visit_cap; ++i) order[i] = EMPTY_ID;
    }
    if constexpr (P <= 2) {
        if (p.rr_ticket) publish_list(p, q, lane);
    }
}

template <int ENC, int NW_T, int G, int P, bool NARROW, bool SPLIT = false>
static hipError_t launch_one(const SearchParams& p, hipStream_t stream) {
    size_t lds = beam_search_lds_bytes(p.nw, p.vis_slots, NARROW, p.ef);
    auto kern = beam_search_kernel<ENC, NW_T, G, P, NARROW, SPLIT>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const bool two_roles = P <= 2 && p.rr_ticket != nullptr;
    hipLaunchKernelGGL(kern, dim3((unsigned)(two_roles ? 2 * p.nq : p.nq)), dim3(64), lds, stream, p);
    return hipGetLastError();
}

template <int ENC, int NW_T, int G, int P>
static hipError_t launch_n(const SearchParams& p, hipStream_t stream) {
    if (p.codes1) {   // rows in the split layout: compiled for the Sign-Magnitude widths and lanes per row kernels.h names
        if constexpr (ENC == ENC_SM && NW_T > 0 && split_lanes_per_row(NW_T) == G)
            return p.vis_regions > 0 ? launch_one<ENC, NW_T, G, P, true, true>(p, stream)
                                     : launch_one<ENC, NW_T, G, P, false, true>(p, stream);
        else
            return hipErrorInvalidValue;
    }
    return p.vis_regions > 0 ? launch_one<ENC, NW_T, G, P, true>(p, stream) : launch_one<ENC, NW_T, G, P, false>(p, stream);
}

template <int ENC, int NW_T, int G>
static hipError_t launch_p(const SearchParams& p, hipStream_t stream) {
    int P = (p.ef + 63) / 64;
    if (P <= 1) return launch_n<ENC, NW_T, G, 1>(p, stream);
    if (P <= 2) return launch_n<ENC, NW_T, G, 2>(p, stream);
    if (P <= 4) return launch_n<ENC, NW_T, G, 4>(p, stream);
    if (P <= 8) return launch_n<ENC, NW_T, G, 8>(p, stream);
    return launch_n<ENC, NW_T, G, 16>(p, stream);
}

template <int ENC, int NW_T>
static hipError_t launch_g(const SearchParams& p, int g, hipStream_t stream) {
    // the ablation encodings at widths other than 768-d are compiled for one gather width only, the one picked by default
    if constexpr (ENC != ENC_SM && NW_T != 0 && NW_T != 12) {
        constexpr int GD = NW_T <= 12 ? 2 : (NW_T <= 32 ? 4 : 16);
        return launch_p<ENC, NW_T, GD>(p, stream);
    }
    switch (g) {
        case 1: return launch_p<ENC, NW_T, 1>(p, stream);
        case 2: return launch_p<ENC, NW_T, 2>(p, stream);
        case 4: return launch_p<ENC, NW_T, 4>(p, stream);
        case 8: return launch_p<ENC, NW_T, 8>(p, stream);
        case 16: return launch_p<ENC, NW_T, 16>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

#if QV_SEARCH_WIDTH == 0 && QV_SEARCH_ENC == 0
static int default_lanes_per_row(int nw) {
    if (nw <= 12) return 2;
    if (nw <= 32) return 4;   // 2048-d: 1.69 ms with 4 lanes per row against 2.02 with 16 (400k vectors, ef = 64)
    return 16;
}

// Launch order.  A batch is a few rounds of resident waves deep, queries differ in length (47 to 157 expansions
// at 1M x 768, ef = 64) and the kernel ends when the last query does, so the long ones should start first.
// How long a query will run is not known, but it grows with the distance between the query's code and the
// entry node's code (rank correlation 0.3-0.4 on the workloads here), which costs one distance per query.
// Each workgroup ranks its 512 queries by that distance (farthest = rank 0, by counting) and the ranks of all
// workgroups are interleaved: launch position = rank * workgroups + workgroup.  Workgroups hold arbitrary
// slices of the batch, so this is the sorted order up to the difference between their quantiles, without any
// global pass.  Only the order in which queries are picked up changes; their outputs go where they always go.
constexpr int ORDER_BLOCK = 512;

__global__ __launch_bounds__(ORDER_BLOCK) void query_order_kernel(const uint64_t* __restrict__ qcodes,
                                                                  const uint64_t* __restrict__ codes, int64_t nq, int nw,
                                                                  int encoding, uint32_t entry, int row_stride,
                                                                  uint32_t* __restrict__ order,
                                                                  uint32_t* __restrict__ rr_ticket,
                                                                  uint32_t* __restrict__ rr_done) {
    __shared__ uint32_t keys[ORDER_BLOCK];
    const int tid = threadIdx.x;
    const int64_t q = (int64_t)blockIdx.x * ORDER_BLOCK + tid;
    if (rr_done && q < nq) rr_done[q] = 0;       // state of a launch with Stage 2 in other waves: no list ready,
    if (rr_ticket && q == 0) *rr_ticket = 0;     // no tickets taken
    if (!order) return;                           // (uniform) a small batch: only that state is wanted
    uint32_t key = (uint32_t)(ORDER_BLOCK - 1 - tid);           // beyond the batch: below every real key
    if (q < nq) {
        const int rw = code_row_words_dev(nw, encoding);
        const uint64_t* ce = codes + (int64_t)entry * row_stride;
        const uint64_t* cq = qcodes + q * rw;
        uint32_t c1 = 0, c2 = 0, c3 = 0;
        for (int w = 0; w < nw; ++w) {
            if (encoding == ENC_SIGN1) {
                c1 += __popcll(cq[w] ^ ce[w]);
            } else if (encoding == ENC_SQ2) {
                const uint64_t la = cq[w], ha = cq[nw + w], lb = ce[w], hb = ce[nw + w];
                c1 += __popcll((la | ha) ^ (lb | hb)) + __popcll((la & ha) ^ (lb & hb));
                c2 += __popcll(ha ^ hb);
            } else {
                const uint64_t X = cq[w] ^ ce[w], sa = cq[nw + w], sb = ce[nw + w];
                c1 += __popcll(X);
                c2 += __popcll(X & (sa | sb));
                c3 += __popcll(X & sa & sb);
            }
        }
        key = ((c1 + c2 + 2u * c3 + 1u) << 9) | key;            // distances stay below 2^19, so 32 bits hold this
    }
    keys[tid] = key;
    __syncthreads();
    uint32_t rank = 0;                                          // keys are distinct: the low bits are the lane's own
    for (int j = 0; j < ORDER_BLOCK; ++j) rank += keys[j] > key ? 1u : 0u;
    if (q >= nq) return;
    const int64_t blocks = gridDim.x, last_valid = nq - (blocks - 1) * ORDER_BLOCK;   // queries in the last workgroup
    const int64_t pos = (int64_t)rank < last_valid ? (int64_t)rank * blocks + blockIdx.x
                                                   : last_valid * blocks + ((int64_t)rank - last_valid) * (blocks - 1) + blockIdx.x;
    order[pos] = (uint32_t)q;
}

bool launch_query_order(const SearchParams& p, uint32_t* order, uint32_t* rr_ticket, uint32_t* rr_done, hipStream_t stream,
                        hipError_t* err) {
    *err = hipSuccess;
    // fewer queries than resident waves all start at once; very large batches amortise their tail
    const bool ordered = p.nq >= 4096 && p.nq <= (1 << 20);
    if (!ordered && !rr_ticket) return false;
    hipLaunchKernelGGL(query_order_kernel, dim3((unsigned)((p.nq + ORDER_BLOCK - 1) / ORDER_BLOCK)), dim3(ORDER_BLOCK), 0,
                       stream, p.qcodes, p.codes, p.nq, p.nw, p.encoding, p.entry, p.row_stride, ordered ? order : nullptr,
                       rr_ticket, rr_done);
    *err = hipGetLastError();
    return ordered && *err == hipSuccess;
}

// Picks the visited-table format for `slots` requested slots (rounded up to a multiple of 1024): 16-bit
// entries when every part of the table keeps enough buckets (16 for a table that never forgets, because
// it probes on inside the part; 1 for a cache, which looks at the home bucket only), else 32-bit entries
// (slots rounded up to a power of two).
void plan_visited_table(SearchParams& p, uint32_t slots, bool allow_narrow, bool cache) {
    const uint32_t regions = (uint32_t)((p.n + 65534) / 65535);
    slots = (slots + 1023u) & ~1023u;
    p.vis_cache = cache ? 1 : 0;
    if (allow_narrow && slots / 8 / regions >= (cache ? 1u : 16u)) {
        p.vis_slots = slots;
        p.vis_regions = regions;
        p.vis_region_buckets = slots / 8 / regions;
        p.vis_bucket_bits = 0;
    } else {
        uint32_t pow2 = 1024;
        while (pow2 < slots) pow2 <<= 1;
        p.vis_slots = pow2;
        p.vis_regions = 0;
        p.vis_region_buckets = 0;
        p.vis_bucket_bits = 0;
        while ((4u << p.vis_bucket_bits) < pow2) p.vis_bucket_bits++;
    }
}

#endif

// This file is compiled once per (encoding, code width) pair (-DQV_SEARCH_ENC=e -DQV_SEARCH_WIDTH=w, w = 64-bit
// words per bit-plane, 0 = any width at run time), so that the instantiations build in parallel; each
// object exports launch_beam_search_w<e, w>, and the object for (ENC_SM, 0) also holds the dispatcher and the
// table planner.  The ablation encodings exist for the same widths (every gather width at 12 words = 768-d, the
// paper's ablation, and at 0; the default gather width elsewhere).
#if !defined(QV_SEARCH_WIDTH) || !defined(QV_SEARCH_ENC)
#error "compile with -DQV_SEARCH_ENC=<encoding> -DQV_SEARCH_WIDTH=<words per plane> (see build.py)"
#endif

template <int ENC, int NW_T>
hipError_t launch_beam_search_w(const SearchParams& p, int g, hipStream_t stream) {
    return launch_g<ENC, NW_T>(p, g, stream);
}
template hipError_t launch_beam_search_w<QV_SEARCH_ENC, QV_SEARCH_WIDTH>(const SearchParams& p, int g, hipStream_t stream);

#if QV_SEARCH_WIDTH == 0 && QV_SEARCH_ENC == 0
// plane widths (64-bit words) the Sign-Magnitude search kernel is compiled for; build.py compiles one object per entry
#define QV_SM_WIDTHS(X) X(2) X(4) X(6) X(8) X(12) X(16) X(24) X(32) X(48)
#define QV_EXT_SM(W) extern template hipError_t launch_beam_search_w<ENC_SM, W>(const SearchParams&, int, hipStream_t);
QV_SM_WIDTHS(QV_EXT_SM)
#undef QV_EXT_SM
#define QV_EXT(E, W) extern template hipError_t launch_beam_search_w<E, W>(const SearchParams&, int, hipStream_t);
QV_EXT(ENC_SIGN1, 0) QV_EXT(ENC_SQ2, 0)
#define QV_EXT_S1(W) QV_EXT(ENC_SIGN1, W)
#define QV_EXT_SQ(W) QV_EXT(ENC_SQ2, W)
QV_SM_WIDTHS(QV_EXT_S1) QV_SM_WIDTHS(QV_EXT_SQ)
#undef QV_EXT_S1
#undef QV_EXT_SQ
#undef QV_EXT

int search_compiled_width_at_least(int nw, int encoding) {
    (void)encoding;   // every encoding is compiled for the same widths
    int best = 0;
#define QV_PICK(W) if (best == 0 && W >= nw) best = W;
    QV_SM_WIDTHS(QV_PICK)
#undef QV_PICK
    return best;
}

hipError_t launch_beam_search(const SearchParams& p, int lanes_per_row, hipStream_t stream) {
    if (p.nq == 0) return hipSuccess;
    int g = lanes_per_row > 0 ? lanes_per_row : default_lanes_per_row(p.nw);
    if (g > 16) g = 16;
    if (p.codes1) {
        if (p.encoding != ENC_SM || split_lanes_per_row(p.nw) == 0) return hipErrorInvalidValue;
        g = split_lanes_per_row(p.nw);
    }
    if (p.encoding == ENC_SIGN1) {
        switch (p.nw) {
#define QV_CASE(W) case W: return launch_beam_search_w<ENC_SIGN1, W>(p, g, stream);
            QV_SM_WIDTHS(QV_CASE)
#undef QV_CASE
            default: return launch_beam_search_w<ENC_SIGN1, 0>(p, g, stream);
        }
    }
    if (p.encoding == ENC_SQ2) {
        switch (p.nw) {
#define QV_CASE(W) case W: return launch_beam_search_w<ENC_SQ2, W>(p, g, stream);
            QV_SM_WIDTHS(QV_CASE)
#undef QV_CASE
            default: return launch_beam_search_w<ENC_SQ2, 0>(p, g, stream);
        }
    }
    switch (p.nw) {
#define QV_CASE(W) case W: return launch_beam_search_w<ENC_SM, W>(p, g, stream);
        QV_SM_WIDTHS(QV_CASE)
#undef QV_CASE
        default: return launch_beam_search_w<ENC_SM, 0>(p, g, stream);
    }
}
#endif

}  // namespace qv
