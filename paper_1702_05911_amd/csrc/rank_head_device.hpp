// Head pass of the bin ranking for two tree parts (Sec. 3.2 "Bin Proposal Heuristic", Sec. 4): the first
// 32, 64 or 128 tuples of the order by summed level-2 distance, ranked by ONE wavefront with the keys in
// registers.  Shared by the head kernel (one wavefront per query) and the re-rank kernel (whose first
// wavefront ranks 128 tuples for a query that the head kernel left over, before the workgroup falls
// back to the full ranking).
#pragma once
#include "rank_device.hpp"

namespace pqt {

constexpr int kHeadT = 128;                    // tuples the head pass can rank
constexpr int kHeadPairs = 704;                // pairs (a, b) with (a+1)(b+1) <= 128: 668, in blocks of 64

// ------------------------------------------------------------------------------------------------
// Head pass.  Most queries reach the candidate budget C within the first few dozen tuples of the
// order (the later ones cannot change the result: their runs would start beyond C).  One wavefront
// per query ranks the first 32 tuples exactly, then -- only if their runs do not fill C -- the first
// 64, then the first 128; if that is still not enough it marks the query for the full pass.  Keys
// live in registers: the pairs of the region (a+1)(b+1) <= T1 are taken from a table ordered by that
// product (so the pairs for a smaller T1 are a prefix), sorted in blocks of 64 across the lanes, and
// folded into the T1 smallest.  No workgroup barrier; LDS only holds the two lists.
// ------------------------------------------------------------------------------------------------
struct alignas(16) HeadPairTable {
    uint8_t a[kHeadPairs], b[kHeadPairs];
};
constexpr HeadPairTable make_head_pair_table() {
    HeadPairTable t{};
    int n = 0;
    for (int p = 1; p <= kHeadT; ++p)
        for (int a = 0; a < kHeadT; ++a)
            if (p % (a + 1) == 0 && p / (a + 1) <= kHeadT) {
                t.a[n] = (uint8_t)a;
                t.b[n] = (uint8_t)(p / (a + 1) - 1);
                ++n;
            }
    for (; n < kHeadPairs; ++n) t.a[n] = t.b[n] = 255;
    return t;
}
static __device__ const HeadPairTable kHeadPairTable = make_head_pair_table();

// number of pairs (a, b), a, b >= 0, with (a+1)(b+1) <= t
inline int head_pair_count(int t) {
    int n = 0;
    for (int a = 0; a < t; ++a) n += t / (a + 1);
    return n;
}

struct HeadLds {
    float A[kHeadT], B[kHeadT];
    uint32_t Aid[kHeadT], Bid[kHeadT];
    uint32_t slot[kHeadT];
};

constexpr int kHeadLevels = 3;
struct HeadLevels {
    int T1[kHeadLevels];      // tuples ranked at each level: min(Tn, 32), min(Tn, 64), min(Tn, 128)
    int npairs[kHeadLevels];  // pairs of the region for that many tuples (a prefix of the table)
};

// One level: ranks the first T1 <= 64 * E tuples, probes their slots, and either writes the final run
// list (returns 1), finds that more tuples are needed (returns 0), or -- on the last level -- lists the
// query for the full pass (returns 1).
// carry (E = 1): the 64 smallest keys of the table entries below e_begin, left by the level before
// (+inf when e_begin = 0); the level only looks at the entries from e_begin on and leaves its own 64
// smallest there.  The table is ordered by (a+1)(b+1), so the entries of a smaller T1 are a prefix.
// TO_LDS (the caller is a re-rank workgroup): the counts (runs, candidates) go to res[0..1] instead of
// meta, and a query that needs more tuples is not listed: the level returns 2 and the caller ranks it.
template <int E, bool TO_LDS = false>
__device__ __forceinline__ int head_level(const RankArgs& g, HeadLds& S, int64_t q, int lane, int R1, int T1,
                                          int e_begin, int npairs, int Tn, bool last_level, unsigned long long& carry,
                                          uint32_t* res = nullptr, const uint8_t* tab_a = kHeadPairTable.a,
                                          const uint8_t* tab_b = kHeadPairTable.b) {
    const int T = g.T;
    const uint32_t C = (uint32_t)g.C;
    // ---- the T1 smallest keys (ordered sum bits, a, b) of the region, ascending over (register, lane) ----
    unsigned long long best[E];
#pragma unroll
    for (int r = 0; r < E; ++r) best[r] = ~0ull;
    if (E == 1) best[0] = carry;
    for (int base = e_begin; base < npairs; base += kWave) {
        const int e = base + lane;
        unsigned long long cur[1] = {~0ull};
        if (e < npairs) {
            const unsigned a = tab_a[e], b = tab_b[e];        // (the table in memory, or the caller's copy in LDS)
            if (a < (unsigned)R1 && b < (unsigned)R1)
                cur[0] = ((unsigned long long)mono_key(S.A[a] + S.B[b]) << 32) | (a << 16) | b;
        }
        wave_sort_chunk<1>(cur, lane, 0u);
        if (base == 0) {
            best[0] = cur[0];
        } else {
            // the 64*E smallest of the ascending runs `best` and `cur` (padded with +inf to 64*E keys):
            // minimum against the reversed padded run gives a bitonic sequence; merge it
            const uint32_t rhi = (uint32_t)__builtin_amdgcn_ds_bpermute((63 - lane) << 2, (int)(uint32_t)(cur[0] >> 32));
            const uint32_t rlo = (uint32_t)__builtin_amdgcn_ds_bpermute((63 - lane) << 2, (int)(uint32_t)cur[0]);
            const unsigned long long y = ((unsigned long long)rhi << 32) | rlo;
            best[E - 1] = y < best[E - 1] ? y : best[E - 1];
            wave_merge_chunk<E>(best, lane, 0u, 64u * E);
        }
    }

    if (E == 1) carry = best[0];

    // ---- probe the first T1 tuples ---------------------------------------------------------------
    uint32_t o0[E], len[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const int t = r * kWave + lane;
        o0[r] = 0;
        len[r] = 0;
        if (t < T1) {
            const unsigned r1 = ((unsigned)best[r] >> 16) & 0xffffu, r2 = (unsigned)best[r] & 0xffffu;
            const unsigned long long lin = (unsigned long long)S.Aid[r1] * g.k1k2 + S.Bid[r2];
            const unsigned long long slot = g.hashed ? slot_of_bin(lin, g.H, g.H_inv) : lin;
            o0[r] = g.offsets[slot];
            len[r] = g.offsets[slot + 1] - o0[r];
            S.slot[t] = (uint32_t)slot;
        }
    }
    if (g.hashed) {
        wave_lds_order();
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const int t = r * kWave + lane;
            if (t < T1) {
                const uint32_t mine = S.slot[t];
                for (int u = 0; u < t; ++u)
                    if (S.slot[u] == mine) len[r] = 0;   // proposed earlier in the order
            }
        }
        wave_lds_order();
    }
    uint32_t start[E], total = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const uint32_t incl = wave_inclusive_sum(len[r], lane);
        start[r] = total + incl - len[r];
        total += (uint32_t)__shfl((int)incl, kWave - 1, kWave);
    }
    if (total < C && T1 < Tn) {                          // not enough yet and more tuples exist
        if (!last_level) return 0;
        if (TO_LDS) return 2;
        if (lane == 0) {
            const uint32_t pos = atomicAdd(&g.counters[0], 1u);
            g.order[pos] = (uint32_t)q;
            g.meta[q] = make_uint2(kMetaTodo, pos);          // .y: its place in the list
        }
        return 1;
    }
    uint32_t nruns = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const bool emit = len[r] > 0 && start[r] < C;
        const unsigned long long mask = __ballot(emit);
        if (emit) g.runs[(size_t)q * T + nruns + __popcll(mask & ((1ull << lane) - 1ull))] = make_uint2(o0[r], start[r]);
        nruns += (uint32_t)__popcll(mask);
    }
    if (lane == 0) {
        if (TO_LDS) {
            res[0] = nruns;
            res[1] = total < C ? total : C;
        } else {
            g.meta[q] = make_uint2(nruns, total < C ? total : C);
        }
    }
    return 1;
}

// the two sorted lists of query q into the wavefront's LDS block
__device__ __forceinline__ void head_load_lists(const RankArgs& g, HeadLds& S, int64_t q, int lane, int R1) {
    const int R = g.R;
    for (int e = lane; e < R1; e += kWave) {
        S.A[e] = g.L_d[q * 2 * R + e];
        S.Aid[e] = g.L_id[q * 2 * R + e];
        S.B[e] = g.L_d[q * 2 * R + R + e];
        S.Bid[e] = g.L_id[q * 2 * R + R + e];
    }
    wave_lds_order();
}

}  // namespace pqt
