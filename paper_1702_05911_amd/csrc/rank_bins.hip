// Bin proposal (Sec. 3.2 "Bin Proposal Heuristic", Sec. 4): rank the combinations of the
// per-part sorted level-2 lists by their summed distance -- the order the paper calls optimal
// and re-sorts by on SIFT1B (Sec. 5.1) -- map each rank tuple to its bin number (Eq. 5),
// hash it (modulo H, Sec. 4), drop repeated and empty slots, and lay the surviving runs of
// the inverted lists end to end until the candidate budget C is reached.
//
// The first T tuples of the order (sum, r1, r2) are found without a priority queue: a pair
// (r1, r2) can only be among the first T if (r1+1)(r2+1) <= T, because every pair that is
// component-wise smaller precedes it.  Only that hyperbolic region (about T ln T pairs) is ever
// evaluated.  A head pass (one wavefront per query) ranks the first 32, then 64, then 128 tuples and
// stops as soon as the candidate budget is filled, which it is for nearly every query; the full pass
// handles the rest: if the region fits the sort buffer it is sorted directly, otherwise the T-th
// smallest key is located by a histogram over the key range (keys recomputed on the fly, never
// stored; an exact radix select when the keys tie heavily) and only the T smallest are collected
// and sorted.
#include <algorithm>
#include <cmath>

#include "pqt_host.hpp"
#include "rank_head_device.hpp"

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
    int cap;     // sort buffer: next_pow2(Tcap), at least 64 (with `place` the buffer holds kKeySlack entries more)
    int npair;   // P = 4: length of each of the two pair lists, min(T, R^2)
    int nreg;    // size of the hyperbolic region of the final ranking (P = 2, 4)
    int nreg_pair;   // P = 4: region size of each pair ranking
    int Tmid;    // P = 2: tuples ranked in the first attempt (most queries need far fewer than Tcap)
    int nreg_mid;    // region size for Tmid
    size_t off_keys, off_hist, off_Ld, off_Lid, off_ps, off_pt, off_len, off_slot, off_part,
        off_misc, total;
};

// hashed: slots may repeat (their lengths and numbers go through LDS); 2: the slots tap also wants the numbers
// place: room for placing the keys by bin (the stand-alone kernels; see rank_pairs)
static RankLds rank_layout(int P, int R, int T, int hashed, bool place) {
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
    L.off_keys = o;  o += sizeof(unsigned long long) * (L.cap + (place ? kKeySlack : 0));
    L.off_hist = o;  o += sizeof(uint32_t) * (place ? kPlaceBins : kSelBins);
    L.off_Ld = o;    o += sizeof(float) * P * R;
    L.off_Lid = o;   o += sizeof(uint32_t) * P * R;
    L.off_ps = o;    o += sizeof(float) * 2 * L.npair;        // summed distances of the two pair lists
    L.off_pt = o;    o += sizeof(uint32_t) * 2 * L.npair;     // their rank pairs (r << 16 | r')
    L.off_len = o;   o += hashed == 1 ? sizeof(uint32_t) * L.Tcap : 0;
    L.off_slot = o;  o += hashed ? sizeof(uint32_t) * L.Tcap : 0;
    L.off_part = o;  o += sizeof(uint32_t) * 32;               // two prefix sums x up to 16 wavefronts
    L.off_misc = o;  o += sizeof(uint32_t) * 16;
    L.total = o;
    return L;
}

size_t rank_lds_bytes(int P, int R, int T, int hashed) { return rank_layout(P, R, T, hashed, true).total; }


__global__ __launch_bounds__(kRankHeadThreads) void rank_head_kernel(RankArgs g, int Tn, HeadLevels lv) {
    __shared__ HeadLds lds[kRankHeadThreads / kWave];
    __shared__ __align__(4) uint8_t tab_a[kHeadPairs], tab_b[kHeadPairs];      // the pair table: one load per thread
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t q = (int64_t)blockIdx.x * (kRankHeadThreads / kWave) + wave;
    static_assert(kHeadPairs % 4 == 0 && kHeadPairs / 4 <= kRankHeadThreads, "a word of each table half per thread");
    if (threadIdx.x < kHeadPairs / 4) {
        reinterpret_cast<uint32_t*>(tab_a)[threadIdx.x] = reinterpret_cast<const uint32_t*>(kHeadPairTable.a)[threadIdx.x];
        reinterpret_cast<uint32_t*>(tab_b)[threadIdx.x] = reinterpret_cast<const uint32_t*>(kHeadPairTable.b)[threadIdx.x];
    }
    HeadLds& S = lds[wave];
    const int R1 = g.R < kHeadT ? g.R : kHeadT;
    if (q < g.nq) head_load_lists(g, S, q, lane, R1);
    __syncthreads();
    if (q >= g.nq) return;
    // levels whose tuple count does not grow are skipped (T smaller than 64 or 128)
    unsigned long long carry = ~0ull;
    if (head_level<1>(g, S, q, lane, R1, lv.T1[0], 0, lv.npairs[0], Tn, lv.T1[1] == lv.T1[0], carry, nullptr, tab_a, tab_b)) return;
    // the second level adds the table entries between the two regions to the 64 smallest of the first
    if (head_level<1>(g, S, q, lane, R1, lv.T1[1], lv.npairs[0], lv.npairs[1], Tn, lv.T1[2] == lv.T1[1], carry, nullptr, tab_a, tab_b))
        return;
    head_level<2>(g, S, q, lane, R1, lv.T1[2], 0, lv.npairs[2], Tn, true, carry, nullptr, tab_a, tab_b);
}

// ------------------------------------------------------------------------------------------------
// Full pass: workgroups take the queries the head pass listed (or every query when forced).
// ------------------------------------------------------------------------------------------------

// MAXPER: tuples a thread may have to hold (T <= MAXPER * kRankThreads).  The variant for at most four is
// compiled for 64 registers, so that two workgroups fit a compute unit: the pass is a chain of dependent
// steps with many barriers, and a second resident query hides most of them.
// PF: the number of tree parts when it is compiled in (4), 0: read from the arguments.
template <int MAXPER, int PF = 0, int MODE = kRankPlace>
__global__ __launch_bounds__(PF == 4 && MAXPER <= 4 ? kRankThreadsFourParts : kRankThreads,
                             MAXPER > 4 ? 4 : (PF == 4 ? 6 : 8)) void rank_kernel(RankArgs g, RankOffsets L) {
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t count = L.force ? (uint32_t)g.nq : g.counters[0];
    for (uint32_t item = blockIdx.x; item < count; item += gridDim.x) {
        const int64_t q = L.force ? (int64_t)item : (int64_t)g.order[item];
        rank_query<PF, false, MAXPER, MODE>(g, L, q, smem, nullptr);
    }
}

// ------------------------------------------------------------------------------------------------
// Fixed traversal order (Sec. 3.2 "Bin Proposal Heuristic": pre-computed orders for ten slopes
// 1.08^k instead of the order by summed distance).  The paper prints neither the weighted norm nor
// the rule that picks a slope; here the order for slope s ranks the pairs v = (v1, v2), counted from
// 1, by v1^2 + (s v2)^2 (ties by (v1, v2)), and a query takes the slope nearest (geometrically) to
// g2 / g1, g_p = L_p[min(R-1, 8)] - L_p[0]: the list that rises more slowly is advanced faster.
// One wavefront per query walks its table 64 tuples at a time and stops when the runs fill C.
// ------------------------------------------------------------------------------------------------
constexpr int kStaticThreads = 256;
constexpr int kSlopeReferenceRank = 8;

__global__ __launch_bounds__(kStaticThreads) void rank_static_kernel(RankArgs g, StaticOrder so) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t q = (int64_t)blockIdx.x * (kStaticThreads / kWave) + threadIdx.x / kWave;
    if (q >= g.nq) return;
    const int R = g.R, T = g.T;
    const uint32_t C = (uint32_t)g.C;
    const float* L1 = g.L_d + q * 2 * R;
    const float* L2 = L1 + R;
    const uint32_t* I1 = g.L_id + q * 2 * R;
    const uint32_t* I2 = I1 + R;
    const int r0 = R - 1 < kSlopeReferenceRank ? R - 1 : kSlopeReferenceRank;
    const float g1 = L1[r0] - L1[0], g2 = L2[r0] - L2[0];
    int k = 0;
#pragma unroll
    for (int j = 0; j < kStaticSlopes - 1; ++j) k += (g2 > so.thr[j] * g1) ? 1 : 0;
    const uint32_t* tab = so.table + (size_t)k * so.Tn;
    const bool every_tuple = g.tuples || g.tuple_keys || g.n_tuples;      // taps want them all
    uint32_t total = 0, nruns = 0;
    for (int base = 0; base < so.Tn; base += kWave) {
        const int t = base + lane;
        uint32_t len = 0, o0 = 0;
        unsigned long long slot = 0;
        if (t < so.Tn) {
            const uint32_t ab = tab[t];
            const uint32_t a = ab >> 16, b = ab & 0xffffu;
            slot = (unsigned long long)I1[a] * g.k1k2 + I2[b];
            o0 = g.offsets[slot];
            len = g.offsets[slot + 1] - o0;
            if (g.tuples) {
                uint16_t* tp = g.tuples + ((size_t)q * T + t) * 4;
                tp[0] = (uint16_t)a; tp[1] = (uint16_t)b; tp[2] = 0; tp[3] = 0;
            }
            if (g.tuple_keys) g.tuple_keys[(size_t)q * T + t] = L1[a] + L2[b];
        }
        const uint32_t incl = wave_inclusive_sum(len, lane);
        const uint32_t start = total + incl - len;
        const bool emit = len > 0 && start < C;
        const unsigned long long mask = __ballot(emit);
        if (emit) {
            const uint32_t idx = nruns + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
            g.runs[(size_t)q * T + idx] = make_uint2(o0, start);
            if (g.slots) g.slots[(size_t)q * T + idx] = slot;
        }
        nruns += (uint32_t)__popcll(mask);
        total += (uint32_t)__shfl((int)incl, kWave - 1, kWave);
        if (total >= C && !every_tuple) break;                  // same for the whole wavefront
    }
    if (lane == 0) {
        g.meta[q] = make_uint2(nruns, total < C ? total : C);
        if (g.n_tuples) g.n_tuples[q] = (uint32_t)so.Tn;
    }
}

int make_static_order(int R, int T, std::vector<uint32_t>& table, float thr[kStaticSlopes - 1]) {
    static_assert(kStaticSlopes == pqt_host::kSlopes, "one table per slope");
    return pqt_host::make_static_order(R, T, table, thr);
}

hipError_t launch_rank_static(const RankArgs& a, const StaticOrder& so, hipStream_t s) {
    if (a.nq <= 0) return hipSuccess;
    if (a.P != 2 || a.hashed || !so.table || so.Tn < 1 || so.Tn > a.T) return hipErrorInvalidValue;
    constexpr int per = kStaticThreads / kWave;
    hipLaunchKernelGGL(rank_static_kernel, dim3((unsigned)((a.nq + per - 1) / per)), dim3(kStaticThreads), 0, s, a, so);
    return hipGetLastError();
}

RankOffsets rank_offsets(int P, int R, int T, int hashed, bool place) {
    const RankLds L = rank_layout(P, R, T, hashed, place);
    RankOffsets o;
    o.Tcap = L.Tcap; o.cap = L.cap; o.npair = L.npair; o.nreg = L.nreg; o.nreg_pair = L.nreg_pair;
    o.Tmid = L.Tmid; o.nreg_mid = L.nreg_mid;
    o.force = 0;
    o.keys = (uint32_t)L.off_keys; o.hist = (uint32_t)L.off_hist;
    o.Ld = (uint32_t)L.off_Ld; o.Lid = (uint32_t)L.off_Lid; o.ps = (uint32_t)L.off_ps; o.pt = (uint32_t)L.off_pt;
    o.len = (uint32_t)L.off_len; o.slot = (uint32_t)L.off_slot;
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
    RankOffsets o = rank_offsets(a.P, a.R, a.T, a.hashed ? 1 : (a.slots ? 2 : 0), true);
    const bool head = rank_has_head(a);
    if (defer_full && !head) return hipErrorInvalidValue;
    o.force = head ? 0 : 1;
    if (head) {
        constexpr int per = kRankHeadThreads / kWave;
        HeadLevels lv;
        for (int l = 0; l < kHeadLevels; ++l) {
            const int t = kHeadT >> (kHeadLevels - 1 - l);          // 32, 64, 128
            lv.T1[l] = o.Tcap < t ? o.Tcap : t;
            lv.npairs[l] = head_pair_count(lv.T1[l]);
        }
        if (defer_full) {
            // the re-rank workgroups rank what is left in full: the third level, one long chain of dependent
            // steps in a single wavefront for a few queries, would only set the duration of this kernel
            lv.T1[2] = lv.T1[1];
            lv.npairs[2] = lv.npairs[1];
        }
        hipLaunchKernelGGL(rank_head_kernel, dim3((unsigned)((a.nq + per - 1) / per)), dim3(kRankHeadThreads), 0, s, a,
                           o.Tcap, lv);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || defer_full) return e;
    }
    const unsigned grid = head ? (unsigned)(a.nq < 1024 ? a.nq : 1024) : (unsigned)a.nq;
    // Four tree parts: the pass is a chain of dependent steps, so what counts is how many queries a compute
    // unit works on at once: workgroups of 512 threads (their LDS lets three share a compute unit, which is
    // also what the kernel's register budget is set for) as long as a thread then holds at most eight tuples.
    if (a.P == 4) {
        const int threads = o.Tcap <= 8 * kRankThreadsFourParts ? kRankThreadsFourParts : kRankThreads;
        if (o.Tcap <= 4 * kRankThreadsFourParts)
            hipLaunchKernelGGL((rank_kernel<4, 4>), dim3(grid), dim3(threads), o.total, s, a, o);
        else
            hipLaunchKernelGGL((rank_kernel<8, 4>), dim3(grid), dim3(threads), o.total, s, a, o);
    } else if (o.Tcap <= 4 * kRankThreads) hipLaunchKernelGGL(rank_kernel<4>, dim3(grid), dim3(kRankThreads), o.total, s, a, o);
    else hipLaunchKernelGGL(rank_kernel<8>, dim3(grid), dim3(kRankThreads), o.total, s, a, o);
    return hipGetLastError();
}

hipError_t configure_rank(size_t max_dynamic_lds) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(rank_kernel<4>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(rank_kernel<4, 4>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)max_dynamic_lds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(rank_kernel<8, 4>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)max_dynamic_lds);
    if (e != hipSuccess) return e;

    return hipFuncSetAttribute(reinterpret_cast<const void*>(rank_kernel<8>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
}

}  // namespace pqt
