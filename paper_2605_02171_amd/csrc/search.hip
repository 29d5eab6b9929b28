// Stage 1 of the query path (paper Sec. 3.3): greedy best-first beam search over a fixed-degree
// graph, navigating only with the symmetric Sign-Magnitude distance of Sec. 3.1 / Table 1.
//
// Mapping to gfx950: one 64-lane wavefront per query, one wavefront per workgroup.
//   * candidate list ("pool"): ef sorted 64-bit keys held in registers, entry e in lane e%64,
//     register e/64.  key = dist << 33 | id << 1 | expanded, so integer order is (dist, id) order.
//   * visited set: exact open-addressing table of 32-bit ids in LDS (linear probing, LDS
//     compare-and-swap).  When it is nearly full it stops taking new ids; from then on a node may
//     be evaluated twice, which cannot change the list (see the note at merge_key) and is reported
//     in the status word.
//   * expansion: lane j reads adj[u][j] (one coalesced row), lanes filter their ids through the
//     visited table, survivors are compacted into LDS, then G lanes cooperate on one neighbour's
//     code: lane s of a group loads words s, s+G, ... of both bit-planes (8*G contiguous bytes
//     per group per load instruction), XOR/AND/OR + popcount, and a G-lane butterfly adds the
//     partial sums.  64/G neighbours are in flight per pass.
//   * merge: new keys below the current worst are inserted one by one with a ballot rank and a
//     one-lane shift.  The pool after an expansion is the ef smallest keys of (old pool U new
//     keys), which does not depend on insertion order, so expanding all neighbours at once
//     reproduces the sequential algorithm exactly.
#include <hip/hip_runtime.h>
#include <stdint.h>

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

__device__ __forceinline__ uint64_t shfl_up1_64(uint64_t v) {
    uint32_t lo = (uint32_t)__shfl_up((int)(uint32_t)v, 1);
    uint32_t hi = (uint32_t)__shfl_up((int)(uint32_t)(v >> 32), 1);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint32_t hash_slot(uint32_t v, int bits) { return (v * 2654435761u) >> (32 - bits); }

// Insert id v (or only look it up when !may_insert).  Returns true when v was not in the table.
__device__ __forceinline__ bool visited_test_and_set(uint32_t* tab, uint32_t mask, int bits, uint32_t v,
                                                     bool may_insert) {
    uint32_t h = hash_slot(v, bits);
    for (;;) {
        uint32_t cur = may_insert ? atomicCAS(&tab[h], EMPTY_ID, v) : tab[h];
        if (cur == EMPTY_ID) return true;   // was free: v is new (and now stored if may_insert)
        if (cur == v) return false;
        h = (h + 1) & mask;                 // the table is never allowed to fill up, so this ends
    }
}

template <int P>
struct Pool {
    uint64_t key[P];
    int size;
};

// Insert one key into the sorted pool (wave-uniform arguments).  A key whose (dist, id) is already
// present is dropped: that only happens after the visited table stopped taking ids, and then a
// re-evaluated node is either still in the pool (dropped here) or was rejected/evicted before, in
// which case it is above the current worst key (the worst key never grows once the pool is full)
// and never reaches this function.
template <int P>
__device__ __forceinline__ void merge_key(Pool<P>& pool, uint64_t nk, int ef, int lane, bool check_dup) {
    int pos = 0;
    bool dup = false;
#pragma unroll
    for (int r = 0; r < P; ++r) {
        pos += __popcll(__ballot(pool.key[r] < nk));
        if (check_dup) dup |= (pool.key[r] >> 1) == (nk >> 1);
    }
    if (check_dup && __any(dup)) return;
    if (pos >= ef) return;
#pragma unroll
    for (int r = P - 1; r >= 0; --r) {
        uint64_t up = shfl_up1_64(pool.key[r]);
        if (r > 0) {
            uint64_t carry = readlane64(pool.key[r - 1], 63);
            if (lane == 0) up = carry;
        }
        int e = r * 64 + lane;
        if (e == pos) pool.key[r] = nk;
        else if (e > pos) pool.key[r] = up;   // lane 0 of register 0 is never > pos unless pos < 0
    }
    if (pool.size < ef) pool.size++;
    // entries at index >= ef are not part of the pool
    if ((ef & 63) || ef < 64 * P) {
#pragma unroll
        for (int r = 0; r < P; ++r)
            if (r * 64 + lane >= ef) pool.key[r] = KEY_NONE;
    }
}

template <int NW_T, int G, int P>
__global__ __launch_bounds__(64) void beam_search_kernel(SearchParams p) {
    extern __shared__ __align__(16) uint32_t smem[];
    const int lane = threadIdx.x;
    const int64_t q = blockIdx.x;
    const int NW = NW_T > 0 ? NW_T : p.nw;
    const int hbits = p.hash_bits;
    const uint32_t cap = 1u << hbits, hmask = cap - 1;
    const uint32_t vis_limit = cap - (cap >> 3) - 64;  // stop inserting at 7/8 full
    uint32_t* tab = smem;
    uint32_t* list = tab + cap;       // [64] compacted new neighbour ids
    uint32_t* dlist = list + 64;      // [64] their distances
    uint64_t* qlds = reinterpret_cast<uint64_t*>(dlist + 64);  // [2*NW] query code (generic path)

    for (uint32_t i = lane; i < cap; i += 64) tab[i] = EMPTY_ID;

    constexpr int RPP = 64 / G;                       // neighbour rows per pass
    constexpr int KW = NW_T > 0 ? (NW_T + G - 1) / G : 1;
    const int sub = lane % G, grp = lane / G;
    const uint64_t* qsrc = p.qcodes + q * (int64_t)(2 * NW);
    uint64_t qp[KW], qs[KW];
    if constexpr (NW_T > 0) {
#pragma unroll
        for (int i = 0; i < KW; ++i) {
            int w = sub + i * G;
            qp[i] = w < NW_T ? qsrc[w] : 0ull;
            qs[i] = w < NW_T ? qsrc[NW_T + w] : 0ull;
        }
    } else {
        for (int w = lane; w < 2 * NW; w += 64) qlds[w] = qsrc[w];
        qp[0] = qs[0] = 0;
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
        for (int base = 0; base < m; base += RPP) {
            int ri = base + grp;
            uint32_t c1 = 0, c2 = 0, c3 = 0;
            if (ri < m) {
                const uint64_t* row = p.codes + (int64_t)list[ri] * (2 * NW);
                if constexpr (NW_T > 0) {
                    uint64_t pv[KW], sv[KW];
#pragma unroll
                    for (int i = 0; i < KW; ++i) {
                        int w = sub + i * G;
                        pv[i] = w < NW_T ? row[w] : 0ull;
                        sv[i] = w < NW_T ? row[NW_T + w] : 0ull;
                    }
#pragma unroll
                    for (int i = 0; i < KW; ++i) {
                        uint64_t X = pv[i] ^ qp[i];
                        c1 += __popcll(X);
                        c2 += __popcll(X & (sv[i] | qs[i]));
                        c3 += __popcll(X & sv[i] & qs[i]);
                    }
                } else {
                    for (int w = sub; w < NW; w += G) {
                        uint64_t X = row[w] ^ qlds[w];
                        uint64_t sv = row[NW + w], sq = qlds[NW + w];
                        c1 += __popcll(X);
                        c2 += __popcll(X & (sv | sq));
                        c3 += __popcll(X & sv & sq);
                    }
                }
            }
            uint32_t dist = c1 + c2 + 2u * c3;
#pragma unroll
            for (int off = G >> 1; off >= 1; off >>= 1) dist += __shfl_xor((int)dist, off);
            if (sub == 0 && ri < m) dlist[ri] = dist;
        }
        wave_sync();
        n_eval += (uint32_t)m;
        uint64_t mine = KEY_NONE;
        if (lane < m) mine = ((uint64_t)dlist[lane] << 33) | ((uint64_t)list[lane] << 1);
        // worst key currently in a full pool; KEY_NONE while there is room
        uint64_t worst = KEY_NONE;
#pragma unroll
        for (int r = 0; r < P; ++r)
            if (r == ((ef - 1) >> 6)) worst = readlane64(pool.key[r], (ef - 1) & 63);
        uint64_t todo = __ballot(mine < worst);
        while (todo) {
            int j = __ffsll((unsigned long long)todo) - 1;
            todo &= todo - 1;
            uint64_t nk = readlane64(mine, j);
            merge_key<P>(pool, nk, ef, lane, vis_full);
        }
    };

    // the entry node
    if (lane == 0) {
        list[0] = p.entry;
        visited_test_and_set(tab, hmask, hbits, p.entry, true);
    }
    n_vis = 1;
    process_list(1);

    for (;;) {
        // best unexpanded entry
        uint32_t uid = EMPTY_ID;
        bool found = false;
#pragma unroll
        for (int r = 0; r < P; ++r) {
            if (!found) {
                uint64_t open = __ballot(pool.key[r] != KEY_NONE && !(pool.key[r] & 1ull));
                if (open) {
                    int l = __ffsll((unsigned long long)open) - 1;
                    uid = (uint32_t)(readlane64(pool.key[r], l) >> 1);
                    if (lane == l) pool.key[r] |= 1ull;
                    found = true;
                }
            }
        }
        if (!found) break;
        if (order && lane == 0 && (int64_t)n_exp < p.visit_cap) order[n_exp] = uid;
        n_exp++;

        const uint32_t* arow = p.adj + (int64_t)uid * p.R;
        for (int c = 0; c < p.R; c += 64) {
            uint32_t v = (c + lane < p.R) ? arow[c + lane] : EMPTY_ID;
            bool valid = v != EMPTY_ID;
            if (valid && (int64_t)v >= p.n) { valid = false; status |= QV_STATUS_BAD_EDGE_BIT; }
            int n_valid = __popcll(__ballot(valid));
            if (!vis_full && n_vis + (uint32_t)n_valid > vis_limit) {
                vis_full = true;
                status |= QV_STATUS_VISITED_FULL_BIT;
            }
            bool fresh = valid && visited_test_and_set(tab, hmask, hbits, v, !vis_full);
            // (with a full table two lanes holding the same id both count as new here; the
            // duplicate check at merge time drops the second one)
            uint64_t fm = __ballot(fresh);
            int m = __popcll(fm);
            if (m == 0) continue;
            if (!vis_full) n_vis += (uint32_t)m;
            wave_sync();  // previous readers of list[] are done
            if (fresh) list[__popcll(fm & ((1ull << lane) - 1ull))] = v;
            process_list(m);
        }
    }

    // results: sorted list, counters
    uint32_t* cid = p.cand_ids + q * (int64_t)ef;
    uint32_t* cds = p.cand_dist + q * (int64_t)ef;
#pragma unroll
    for (int r = 0; r < P; ++r) {
        int e = r * 64 + lane;
        if (e < ef) {
            bool has = pool.key[r] != KEY_NONE;
            cid[e] = has ? (uint32_t)(pool.key[r] >> 1) : EMPTY_ID;
            cds[e] = has ? (uint32_t)(pool.key[r] >> 33) : EMPTY_ID;
        }
    }
    status = (uint32_t)__builtin_amdgcn_readfirstlane((int)status) |
             (__any(status & QV_STATUS_BAD_EDGE_BIT) ? QV_STATUS_BAD_EDGE_BIT : 0u);
    if (lane == 0) {
        p.n_cand[q] = (uint32_t)pool.size;
        if (p.n_expanded) p.n_expanded[q] = n_exp;
        if (p.n_evals) p.n_evals[q] = n_eval;
        if (p.status) p.status[q] = status;
        if (order)
            for (int64_t i = n_exp; i < p.visit_cap; ++i) order[i] = EMPTY_ID;
    }
}

size_t beam_search_lds_bytes(int nw, int hash_bits) {
    return ((size_t)1 << hash_bits) * 4 + 64 * 4 * 2 + (size_t)nw * 16 + 16;
}

template <int NW_T, int G, int P>
static hipError_t launch_one(const SearchParams& p, hipStream_t stream) {
    size_t lds = beam_search_lds_bytes(p.nw, p.hash_bits);
    auto kern = beam_search_kernel<NW_T, G, P>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)p.nq), dim3(64), lds, stream, p);
    return hipGetLastError();
}

template <int NW_T, int G>
static hipError_t launch_p(const SearchParams& p, hipStream_t stream) {
    int P = (p.ef + 63) / 64;
    if (P <= 1) return launch_one<NW_T, G, 1>(p, stream);
    if (P <= 2) return launch_one<NW_T, G, 2>(p, stream);
    if (P <= 4) return launch_one<NW_T, G, 4>(p, stream);
    if (P <= 8) return launch_one<NW_T, G, 8>(p, stream);
    return launch_one<NW_T, G, 16>(p, stream);
}

template <int NW_T>
static hipError_t launch_g(const SearchParams& p, int g, hipStream_t stream) {
    switch (g) {
        case 1: return launch_p<NW_T, 1>(p, stream);
        case 2: return launch_p<NW_T, 2>(p, stream);
        case 4: return launch_p<NW_T, 4>(p, stream);
        case 8: return launch_p<NW_T, 8>(p, stream);
        case 16: return launch_p<NW_T, 16>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

static int default_lanes_per_row(int nw) {
    if (nw <= 2) return 2;
    if (nw <= 6) return 2;
    if (nw <= 12) return 4;
    if (nw <= 24) return 8;
    return 16;
}

hipError_t launch_beam_search(const SearchParams& p, int lanes_per_row, hipStream_t stream) {
    if (p.nq == 0) return hipSuccess;
    int g = lanes_per_row > 0 ? lanes_per_row : default_lanes_per_row(p.nw);
    if (g > 16) g = 16;
    switch (p.nw) {
        case 2: return launch_g<2>(p, g, stream);
        case 6: return launch_g<6>(p, g, stream);
        case 8: return launch_g<8>(p, g, stream);
        case 12: return launch_g<12>(p, g, stream);
        case 48: return launch_g<48>(p, g, stream);
        default: return launch_g<0>(p, g, stream);
    }
}

}  // namespace qv
