// Bin proposal (Sec. 3.2 "Bin Proposal Heuristic", Sec. 4): rank the combinations of the
// per-part sorted level-2 lists by their summed distance -- the order the paper calls optimal
// and re-sorts by on SIFT1B (Sec. 5.1) -- map each rank tuple to its bin number (Eq. 5),
// hash it (modulo H, Sec. 4), drop repeated and empty slots, and lay the surviving runs of
// the inverted lists end to end until the candidate budget C is reached.
//
// The first T tuples of the order (sum, r1, r2) are found without a priority queue: a pair
// (r1, r2) can only be among the first T if (r1+1)(r2+1) <= T, because every pair that is
// component-wise smaller precedes it.  Only that hyperbolic region (about T ln T pairs) is ever
// evaluated.  A head pass (one wavefront per query) ranks the first 64 tuples, which is enough
// for most queries to fill the candidate budget; the full pass handles the rest: if the region
// fits the sort buffer it is sorted directly, otherwise the T-th smallest key is found by a
// radix select over the region (keys recomputed on the fly, never stored) and only the T
// smallest are collected and sorted.
#include "rank_device.hpp"

namespace pqt {

// Number of pairs (a, b), a < nA, b < nB, with (a+1)(b+1) <= Tn.
static long region_size(int nA, int nB, int Tn) {
    long n = 0;
    for (int a = 0; a < nA && a < Tn; ++a) n += region_row_count(a, nB, Tn);
    return n;
}

int rank_region_size(int R, int T) { return (int)region_size(R, R, T); }


struct RankLds {
    int Tcap;    // tuples examined: min(T, R^P)
    int cap;     // sort buffer entries: next_pow2(Tcap), at least 64
    int npair;   // P = 4: length of each of the two pair lists, min(T, R^2)
    int nreg;    // size of the hyperbolic region of the final ranking (P = 2, 4)
    int nreg_pair;   // P = 4: region size of each pair ranking
    int Tmid;    // P = 2: tuples ranked in the first attempt (most queries need far fewer than Tcap)
    int nreg_mid;    // region size for Tmid
    size_t off_keys, off_hist, off_Ld, off_Lid, off_ps, off_pt, off_len, off_o0, off_slot, off_part,
        off_misc, total;
};

static RankLds rank_layout(int P, int R, int T, int hashed) {
    (void)hashed;                      // the de-duplication keys reuse the sort buffer
    RankLds L;
    long total_tuples = 1;
    for (int p = 0; p < P; ++p) total_tuples = (total_tuples * R > (1L << 40)) ? (1L << 40) : total_tuples * R;
    L.Tcap = (int)((long)T < total_tuples ? (long)T : total_tuples);
    L.cap = next_pow2(L.Tcap) < 64 ? 64 : next_pow2(L.Tcap);
    L.npair = 0;
    L.nreg_pair = 0;
    L.Tmid = L.Tcap;
    L.nreg_mid = 0;
    if (P == 1) {
        L.nreg = L.Tcap;
    } else if (P == 2) {
        L.nreg = (int)region_size(R, R, L.Tcap);
        L.Tmid = L.Tcap < kMidT ? L.Tcap : kMidT;
        L.nreg_mid = (int)region_size(R, R, L.Tmid);
    } else {
        L.npair = (int)((long)T < (long)R * R ? (long)T : (long)R * R);
        L.nreg_pair = (int)region_size(R, R, L.npair);
        L.nreg = (int)region_size(L.npair, L.npair, L.Tcap);
    }
    size_t o = 0;
    L.off_keys = o;  o += sizeof(unsigned long long) * L.cap;
    L.off_hist = o;  o += sizeof(uint32_t) * kSelBins;
    L.off_Ld = o;    o += sizeof(float) * P * R;
    L.off_Lid = o;   o += sizeof(uint32_t) * P * R;
    L.off_ps = o;    o += sizeof(float) * 2 * L.npair;        // summed distances of the two pair lists
    L.off_pt = o;    o += sizeof(uint32_t) * 2 * L.npair;     // their rank pairs (r << 16 | r')
    L.off_len = o;   o += sizeof(uint32_t) * L.Tcap;
    L.off_o0 = o;    o += sizeof(uint32_t) * L.Tcap;
    L.off_slot = o;  o += sizeof(uint32_t) * L.Tcap;
    L.off_part = o;  o += sizeof(uint32_t) * 32;               // two prefix sums x up to 16 wavefronts
    L.off_misc = o;  o += sizeof(uint32_t) * 16;
    L.total = o;
    return L;
}

size_t rank_lds_bytes(int P, int R, int T, int hashed) { return rank_layout(P, R, T, hashed).total; }


constexpr int kHeadT = 64;                     // tuples the head pass can rank
constexpr int kHeadPairs = 320;                // pairs (a, b) with (a+1)(b+1) <= 64: 280, in blocks of 64

// ------------------------------------------------------------------------------------------------
// Head pass.  Most queries reach the candidate budget C within the first few dozen tuples of the
// order (the later ones cannot change the result: their runs would start beyond C).  One wavefront
// per query ranks the first 32 tuples exactly, then -- only if their runs do not fill C -- the first
// 64; if that is still not enough it marks the query for the full pass.  Keys live in registers: the
// pairs of the region (a+1)(b+1) <= T1 are taken from a table ordered by that product (so the pairs
// for a smaller T1 are a prefix), sorted in blocks of 64 across the lanes, and folded into the 64
// smallest.  No workgroup barrier; LDS only holds the two lists.
// ------------------------------------------------------------------------------------------------
struct HeadPairTable {
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
__device__ const HeadPairTable kHeadPairTable = make_head_pair_table();

// number of pairs (a, b), a, b >= 0, with (a+1)(b+1) <= t
static int head_pair_count(int t) {
    int n = 0;
    for (int a = 0; a < t; ++a) n += t / (a + 1);
    return n;
}

struct HeadLds {
    float A[kHeadT], B[kHeadT];
    uint32_t Aid[kHeadT], Bid[kHeadT];
    uint32_t slot[kHeadT];
};

struct HeadLevels {
    int T1[2];      // tuples ranked at each level: min(Tn, 32), min(Tn, 64)
    int npairs[2];  // pairs of the region for that many tuples (a prefix of the table)
};

__global__ __launch_bounds__(kRankHeadThreads) void rank_head_kernel(RankArgs g, int Tn, HeadLevels lv) {
    __shared__ HeadLds lds[kRankHeadThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t q = (int64_t)blockIdx.x * (kRankHeadThreads / kWave) + wave;
    if (q >= g.nq) return;
    HeadLds& S = lds[wave];
    const int R = g.R, T = g.T;
    const int R1 = R < kHeadT ? R : kHeadT;
    const uint32_t C = (uint32_t)g.C;

    if (lane < R1) {
        S.A[lane] = g.L_d[q * 2 * R + lane];
        S.Aid[lane] = g.L_id[q * 2 * R + lane];
        S.B[lane] = g.L_d[q * 2 * R + R + lane];
        S.Bid[lane] = g.L_id[q * 2 * R + R + lane];
    }
    wave_lds_order();

    for (int level = 0; level < 2; ++level) {
        const int T1 = lv.T1[level];
        const int npairs = lv.npairs[level];
        // ---- the T1 smallest keys (ordered sum bits, a, b) of the region, ascending over the lanes ----
        unsigned long long best[1] = {~0ull};
        for (int blk = 0; blk * kWave < npairs; ++blk) {
            const int e = blk * kWave + lane;
            unsigned long long cur[1] = {~0ull};
            if (e < npairs) {
                const unsigned a = kHeadPairTable.a[e], b = kHeadPairTable.b[e];
                if (a < (unsigned)R1 && b < (unsigned)R1)
                    cur[0] = ((unsigned long long)mono_key(S.A[a] + S.B[b]) << 32) | (a << 16) | b;
            }
            wave_sort_chunk<1>(cur, lane, 0u);
            if (blk == 0) {
                best[0] = cur[0];
            } else {
                // the 64 smallest of two ascending runs x, y: min(x[i], y[63-i]) is bitonic; merge it
                const uint32_t rhi = (uint32_t)__builtin_amdgcn_ds_bpermute((63 - lane) << 2, (int)(uint32_t)(cur[0] >> 32));
                const uint32_t rlo = (uint32_t)__builtin_amdgcn_ds_bpermute((63 - lane) << 2, (int)(uint32_t)cur[0]);
                const unsigned long long y = ((unsigned long long)rhi << 32) | rlo;
                best[0] = y < best[0] ? y : best[0];
                wave_merge_chunk<1>(best, lane, 0u, 64u);
            }
        }

        // ---- probe the first T1 tuples ---------------------------------------------------------------
        uint32_t o0 = 0, len = 0;
        if (lane < T1) {
            const unsigned r1 = ((unsigned)best[0] >> 16) & 0xffffu, r2 = (unsigned)best[0] & 0xffffu;
            const unsigned long long lin = (unsigned long long)S.Aid[r1] * g.k1k2 + S.Bid[r2];
            const unsigned long long slot = g.hashed ? (lin % g.H) : lin;
            o0 = g.offsets[slot];
            len = g.offsets[slot + 1] - o0;
            S.slot[lane] = (uint32_t)slot;
        }
        if (g.hashed) {
            wave_lds_order();
            if (lane < T1) {
                const uint32_t mine = S.slot[lane];
                for (int t = 0; t < lane; ++t)
                    if (S.slot[t] == mine) len = 0;      // proposed earlier in the order
            }
            wave_lds_order();
        }
        const uint32_t incl_len = wave_inclusive_sum(len, lane);
        const uint32_t start = incl_len - len;
        const uint32_t total = __shfl(incl_len, kWave - 1, kWave);
        if (total < C && T1 < Tn) {                      // not enough yet and more tuples exist
            if (level == 0 && lv.T1[1] > T1) continue;   // rank twice as many
            if (lane == 0) {
                const uint32_t pos = atomicAdd(&g.counters[0], 1u);
                g.order[pos] = (uint32_t)q;
                g.meta[q] = make_uint2(kMetaTodo, pos);      // .y: its place in the list
            }
            return;
        }
        const bool emit = len > 0 && start < C;
        const unsigned long long mask = __ballot(emit);
        if (emit) {
            const int idx = __popcll(mask & ((1ull << lane) - 1ull));
            g.runs[(size_t)q * T + idx] = make_uint2(o0, start);
        }
        if (lane == 0) g.meta[q] = make_uint2((uint32_t)__popcll(mask), total < C ? total : C);
        return;
    }
}

// ------------------------------------------------------------------------------------------------
// Full pass: workgroups take the queries the head pass listed (or every query when forced).
// ------------------------------------------------------------------------------------------------

__global__ __launch_bounds__(kRankThreads) void rank_kernel(RankArgs g, RankOffsets L) {
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t count = L.force ? (uint32_t)g.nq : g.counters[0];
    for (uint32_t item = blockIdx.x; item < count; item += gridDim.x) {
        const int64_t q = L.force ? (int64_t)item : (int64_t)g.order[item];
        rank_query<0, false, 8>(g, L, q, smem, nullptr, nullptr, nullptr);
    }
}

RankOffsets rank_offsets(int P, int R, int T, int hashed) {
    const RankLds L = rank_layout(P, R, T, hashed);
    RankOffsets o;
    o.Tcap = L.Tcap; o.cap = L.cap; o.npair = L.npair; o.nreg = L.nreg; o.nreg_pair = L.nreg_pair;
    o.Tmid = L.Tmid; o.nreg_mid = L.nreg_mid;
    o.force = 0;
    o.keys = (uint32_t)L.off_keys; o.hist = (uint32_t)L.off_hist;
    o.Ld = (uint32_t)L.off_Ld; o.Lid = (uint32_t)L.off_Lid; o.ps = (uint32_t)L.off_ps; o.pt = (uint32_t)L.off_pt;
    o.len = (uint32_t)L.off_len; o.o0 = (uint32_t)L.off_o0; o.slot = (uint32_t)L.off_slot;
    o.part = (uint32_t)L.off_part; o.misc = (uint32_t)L.off_misc;
    o.total = (uint32_t)L.total;
    return o;
}

bool rank_has_head(const RankArgs& a) {
    const bool taps = a.n_tuples || a.tuples || a.tuple_keys || a.slots;
    return a.P == 2 && !taps && a.order && a.counters;
}

hipError_t launch_rank(const RankArgs& a, hipStream_t s, bool defer_full) {
    if (a.nq <= 0) return hipSuccess;
    RankOffsets o = rank_offsets(a.P, a.R, a.T, a.hashed);
    const bool head = rank_has_head(a);
    if (defer_full && !head) return hipErrorInvalidValue;
    o.force = head ? 0 : 1;
    if (head) {
        constexpr int per = kRankHeadThreads / kWave;
        HeadLevels lv;
        lv.T1[0] = o.Tcap < kHeadT / 2 ? o.Tcap : kHeadT / 2;
        lv.T1[1] = o.Tcap < kHeadT ? o.Tcap : kHeadT;
        lv.npairs[0] = head_pair_count(lv.T1[0]);
        lv.npairs[1] = head_pair_count(lv.T1[1]);
        hipLaunchKernelGGL(rank_head_kernel, dim3((unsigned)((a.nq + per - 1) / per)), dim3(kRankHeadThreads), 0, s, a,
                           o.Tcap, lv);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || defer_full) return e;
    }
    const unsigned grid = head ? (unsigned)(a.nq < 1024 ? a.nq : 1024) : (unsigned)a.nq;
    hipLaunchKernelGGL(rank_kernel, dim3(grid), dim3(kRankThreads), o.total, s, a, o);
    return hipGetLastError();
}

hipError_t configure_rank(size_t max_dynamic_lds) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(rank_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
}

}  // namespace pqt
