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
#include "pqt_device.hpp"
#include "pqt_kernels.hpp"

namespace pqt {

__host__ __device__ inline int region_row_count(int a, int R, int T) {
    const int c = T / (a + 1);
    return c < R ? c : R;
}

// Number of pairs (a, b), a < nA, b < nB, with (a+1)(b+1) <= Tn.
static long region_size(int nA, int nB, int Tn) {
    long n = 0;
    for (int a = 0; a < nA && a < Tn; ++a) n += region_row_count(a, nB, Tn);
    return n;
}

int rank_region_size(int R, int T) { return (int)region_size(R, R, T); }

constexpr int kSelBits = 10;
constexpr int kSelBins = 1 << kSelBits;
constexpr int kMidT = 256;         // tuples ranked first by the full pass; all T only if they do not fill C
constexpr int kRegionSplit = 64;   // rows below it are walked along b, the rest of the region along a

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
    L.off_part = o;  o += sizeof(uint32_t) * (kRankThreads + 1);
    L.off_misc = o;  o += sizeof(uint32_t) * 16;
    L.total = o;
    return L;
}

size_t rank_lds_bytes(int P, int R, int T, int hashed) { return rank_layout(P, R, T, hashed).total; }

struct RankOffsets {   // layout handed to the kernel (computed once on the host)
    int Tcap, cap, npair, nreg, nreg_pair, Tmid, nreg_mid;
    int force;             // 1: rank every query (taps wanted, or no head pass ran)
    uint32_t keys, hist, Ld, Lid, ps, pt, len, o0, slot, part, misc;
};

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
            if (lane == 0) g.todo[1 + atomicAdd(&g.todo[0], 1u)] = (uint32_t)q;
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

// Calls f(ordered sum bits, a, b) for every pair of the region {a < nA, b < nB, (a+1)(b+1) <= Tn},
// each pair once, spread over the workgroup.  Rows a < kRegionSplit are walked along b (they are
// long); the remaining pairs have b < Tn / (kRegionSplit + 1) and are walked along a, so lanes stay
// busy in the thin tail of the hyperbola as well.
template <typename F>
__device__ __forceinline__ void for_region(const float* A, int nA, const float* B, int nB, int Tn, int wave,
                                           int lane, F&& f) {
    constexpr int nwaves = kRankThreads / kWave;
    const int rows = min(min(nA, Tn), kRegionSplit);
    for (int a = wave; a < rows; a += nwaves) {
        const int cnt = region_row_count(a, nB, Tn);
        const float da = A[a];
        for (int b = lane; b < cnt; b += kWave) f(mono_key(da + B[b]), (uint32_t)a, (uint32_t)b);
    }
    if (nA > kRegionSplit) {
        const int cols = min(nB, Tn / (kRegionSplit + 1));
        for (int b = wave; b < cols; b += nwaves) {
            const int hi = min(nA, Tn / (b + 1));
            const float db = B[b];
            for (int a = kRegionSplit + lane; a < hi; a += kWave) f(mono_key(A[a] + db), (uint32_t)a, (uint32_t)b);
        }
    }
}

// Appends `key` to keys[] for every lane with take set; one LDS atomic per wavefront instruction.
__device__ __forceinline__ void wave_append(bool take, unsigned long long key, unsigned long long* keys,
                                            uint32_t* counter, int lane) {
    const unsigned long long m = __ballot(take);
    if (!take) return;
    const int leader = __ffsll((long long)m) - 1;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
    base = (uint32_t)__shfl((int)base, leader, kWave);
    keys[base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] = key;
}

// Leaves in keys[0..Tn) the first Tn pairs (a, b) of two ascending lists A[0..nA), B[0..nB) in the
// order (fl32(A[a] + B[b]), a, b), as sorted keys (ordered sum bits << 32 | a << 16 | b).
// Tn <= nA * nB; nreg = size of the region (a+1)(b+1) <= Tn; cap = entries of keys[] (a power of two
// >= Tn).  If the region fits it is sorted directly; otherwise the Tn-th smallest key is found by a
// radix select over the region (sums recomputed in every pass, never stored), ties at that key are cut
// by (a, b), and only the Tn smallest are collected and sorted.  All threads call it; ends with a barrier.
__device__ __forceinline__ void rank_pairs(const float* A, int nA, const float* B, int nB, int Tn, int nreg,
                                           int cap, unsigned long long* keys, uint32_t* hist, uint32_t* misc) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint32_t tau = 0xffffffffu, a_cut = 0xffffffffu, b_cut = 0xffffffffu;
    const bool all = nreg <= cap;
    if (!all) {
        // ---- usual case: one histogram over the range of the region's keys ----------------------------
        // The region's smallest key is A[0]+B[0]; its largest is the last key of some row (both lists
        // ascend).  1024 bins over that range: the bin holding the Tn-th key is found, the
        // keys of lower bins go straight to keys[], the keys of that bin (a handful) to a side buffer
        // that reuses the histogram, is sorted, and gives its first Tn - (lower count).
        constexpr int kTailCap = kSelBins / 2;           // 64-bit entries the histogram's memory holds
        const uint32_t lo_key = mono_key(A[0] + B[0]);
        if (tid < 2) misc[tid] = 0;                      // [0] range maximum, [1] unused here
        for (int e = tid; e < kSelBins; e += kRankThreads) hist[e] = 0;
        __syncthreads();
        {
            const int rows = min(nA, Tn);               // every key of row a is <= the row's last key
            uint32_t kmax = lo_key;
            for (int a = tid; a < rows; a += kRankThreads)
                kmax = max(kmax, mono_key(A[a] + B[region_row_count(a, nB, Tn) - 1]));
            kmax = wave_max_u32(kmax);
            if (lane == 0 && kmax > lo_key) atomicMax(&misc[0], kmax);
        }
        __syncthreads();
        const uint32_t hi_key = max(misc[0], lo_key);
        const uint32_t range = hi_key - lo_key;
        const int width = 32 - __clz((int)(range | 1u));
        const int shift = width > kSelBits ? width - kSelBits : 0;
        for_region(A, nA, B, nB, Tn, wave, lane, [&](uint32_t k32, uint32_t, uint32_t) {
            atomicAdd(&hist[(k32 - lo_key) >> shift], 1u);
        });
        __syncthreads();
        if (tid < kWave) {
            uint32_t bsel, below, inbin;
            hist_locate(hist, (uint32_t)Tn, lane, bsel, below, inbin);
            if (tid == 0) {
                misc[2] = bsel;
                misc[3] = below;
                misc[4] = inbin;
                misc[0] = 0;                             // entries of keys[]
                misc[1] = 0;                             // entries of the side buffer
            }
        }
        __syncthreads();
        const uint32_t bsel = misc[2], below = misc[3], inbin = misc[4];
        if (inbin <= (uint32_t)kTailCap) {
            unsigned long long* tail = reinterpret_cast<unsigned long long*>(hist);
            for_region(A, nA, B, nB, Tn, wave, lane, [&](uint32_t k32, uint32_t a, uint32_t b) {
                const uint32_t bin = (k32 - lo_key) >> shift;
                const unsigned long long key = ((unsigned long long)k32 << 32) | (a << 16) | b;
                wave_append(bin < bsel, key, keys, &misc[0], lane);
                wave_append(bin == bsel, key, tail, &misc[1], lane);
            });
            __syncthreads();
            const int ntail = (int)inbin;
            const int tpad = next_pow2(ntail) < 64 ? 64 : next_pow2(ntail);
            for (int e = ntail + tid; e < tpad; e += kRankThreads) tail[e] = ~0ull;
            block_sort_lds(tail, tpad, tid, kRankThreads);
            for (int e = tid; e < Tn - (int)below; e += kRankThreads) keys[below + e] = tail[e];
            const int npad = next_pow2(Tn);
            for (int e = Tn + tid; e < npad; e += kRankThreads) keys[e] = ~0ull;
            block_sort_lds(keys, npad, tid, kRankThreads);
            return;
        }
        // ---- heavily tied keys: exact radix select ----------------------------------------------------
        __syncthreads();
        uint32_t prefix = 0, mask = 0, need = (uint32_t)Tn, less = 0, neq = 0;
        const int shifts[4] = {22, 12, 2, 0};
        const int nbits[4] = {10, 10, 10, 2};
        for (int pass = 0; pass < 4; ++pass) {
            for (int e = tid; e < kSelBins; e += kRankThreads) hist[e] = 0;
            __syncthreads();
            const int sh = shifts[pass];
            const uint32_t dm = (1u << nbits[pass]) - 1u;
            for_region(A, nA, B, nB, Tn, wave, lane, [&](uint32_t k32, uint32_t, uint32_t) {
                if ((k32 & mask) == prefix) atomicAdd(&hist[(k32 >> sh) & dm], 1u);
            });
            __syncthreads();
            uint32_t digit, before, cnt;
            hist_locate(hist, need, lane, digit, before, cnt);
            less += before;
            need -= before;
            neq = cnt;
            prefix |= digit << sh;
            mask |= dm << sh;
            __syncthreads();
        }
        tau = prefix;                                    // Tn-th smallest sum key; `need` of the neq ties count
        if (less + neq > (uint32_t)cap) {                // too many ties to sort: cut them by (a, b)
            // a and b can exceed the histogram's 1024 bins: select on the high then the low digit
            uint32_t before, cnt, hi_d, lo_d;
            auto pass = [&](auto&& digit_of) {           // digit_of(k32, a, b) -> bin or 0xffffffff (skip)
                for (int e = tid; e < kSelBins; e += kRankThreads) hist[e] = 0;
                __syncthreads();
                for_region(A, nA, B, nB, Tn, wave, lane, [&](uint32_t k32, uint32_t a, uint32_t b) {
                    const uint32_t d = digit_of(k32, a, b);
                    if (d != 0xffffffffu) atomicAdd(&hist[d], 1u);
                });
                __syncthreads();
                uint32_t digit;
                hist_locate(hist, need, lane, digit, before, cnt);
                need -= before;
                __syncthreads();
                return digit;
            };
            hi_d = pass([&](uint32_t k32, uint32_t a, uint32_t) { return k32 == tau ? (a >> 6) : 0xffffffffu; });
            lo_d = pass([&](uint32_t k32, uint32_t a, uint32_t) {
                return (k32 == tau && (a >> 6) == hi_d) ? (a & 63u) : 0xffffffffu;
            });
            a_cut = (hi_d << 6) | lo_d;
            hi_d = pass([&](uint32_t k32, uint32_t a, uint32_t b) {
                return (k32 == tau && a == a_cut) ? (b >> 6) : 0xffffffffu;
            });
            lo_d = pass([&](uint32_t k32, uint32_t a, uint32_t b) {
                return (k32 == tau && a == a_cut && (b >> 6) == hi_d) ? (b & 63u) : 0xffffffffu;
            });
            b_cut = (hi_d << 6) | lo_d;
        }
    }
    if (tid == 0) misc[0] = 0;
    __syncthreads();
    for_region(A, nA, B, nB, Tn, wave, lane, [&](uint32_t k32, uint32_t a, uint32_t b) {
        bool take = all || k32 < tau;
        if (!all && k32 == tau) take = a_cut == 0xffffffffu || a < a_cut || (a == a_cut && b <= b_cut);
        wave_append(take, ((unsigned long long)k32 << 32) | (a << 16) | b, keys, &misc[0], lane);
    });
    __syncthreads();
    const int n = (int)misc[0];
    const int npad = next_pow2(n);
    for (int e = n + tid; e < npad; e += kRankThreads) keys[e] = ~0ull;
    block_sort_lds(keys, npad, tid, kRankThreads);
}

__global__ __launch_bounds__(kRankThreads) void rank_kernel(RankArgs g, RankOffsets L) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem + L.keys);
    unsigned long long* dkeys = keys;                       // (slot, position) keys reuse the sort buffer
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
    float* sLd = reinterpret_cast<float*>(smem + L.Ld);
    uint32_t* sLid = reinterpret_cast<uint32_t*>(smem + L.Lid);
    float* ps = reinterpret_cast<float*>(smem + L.ps);
    uint32_t* pt = reinterpret_cast<uint32_t*>(smem + L.pt);
    uint32_t* slen = reinterpret_cast<uint32_t*>(smem + L.len);
    uint32_t* so0 = reinterpret_cast<uint32_t*>(smem + L.o0);
    uint32_t* sslot = reinterpret_cast<uint32_t*>(smem + L.slot);
    uint32_t* part = reinterpret_cast<uint32_t*>(smem + L.part);
    uint32_t* misc = reinterpret_cast<uint32_t*>(smem + L.misc);

    const int tid = threadIdx.x;
    const int P = g.P, R = g.R, T = g.T;
    const uint32_t C = (uint32_t)g.C;
    const uint32_t count = L.force ? (uint32_t)g.nq : g.todo[0];
    for (uint32_t item = blockIdx.x; item < count; item += gridDim.x) {
        const int64_t q = L.force ? (int64_t)item : (int64_t)g.todo[1 + item];

        for (int e = tid; e < P * R; e += kRankThreads) {
            sLd[e] = g.L_d[q * P * R + e];
            sLid[e] = g.L_id[q * P * R + e];
        }
        __syncthreads();

        // Two attempts for two parts: the first Tmid tuples fill the candidate budget for almost every
        // query (tuples after the one that reaches C cannot change the result); all Tcap otherwise.
        // With taps every tuple is wanted, so only the full attempt runs.
        const bool staged = P == 2 && !L.force && L.Tmid < L.Tcap;
        for (int attempt = staged ? 0 : 1; attempt < 2; ++attempt) {
            const int Tn = attempt == 0 ? L.Tmid : L.Tcap;        // tuples ranked in this attempt

            // ---- the first Tn tuples, sorted, as keys (ordered sum bits, position, position) ---------
            if (P == 1) {
                for (int e = tid; e < Tn; e += kRankThreads)
                    keys[e] = ((unsigned long long)mono_key(sLd[e]) << 32) | (unsigned)e;
                __syncthreads();                 // the list is already sorted by (distance, id)
            } else if (P == 2) {
                rank_pairs(sLd, R, sLd + R, R, Tn, attempt == 0 ? L.nreg_mid : L.nreg, L.cap, keys, hist, misc);
            } else {
                // parts (1,2) and (3,4) first; then pairs of positions in those two lists
                const int np = L.npair;
                for (int half = 0; half < 2; ++half) {
                    rank_pairs(sLd + 2 * half * R, R, sLd + (2 * half + 1) * R, R, np, L.nreg_pair, L.cap, keys, hist,
                               misc);
                    for (int e = tid; e < np; e += kRankThreads) {
                        const unsigned long long key = keys[e];
                        ps[half * np + e] = mono_inv((uint32_t)(key >> 32));
                        pt[half * np + e] = (uint32_t)key;
                    }
                    __syncthreads();
                }
                rank_pairs(ps, np, ps + np, np, Tn, L.nreg, L.cap, keys, hist, misc);
            }

            // ---- tuple -> bin number -> slot -> run of the inverted list ---------------------------
            for (int t = tid; t < Tn; t += kRankThreads) {
                const unsigned long long key = keys[t];
                unsigned long long lin;
                unsigned r[4] = {0, 0, 0, 0};
                if (P == 1) {
                    r[0] = (unsigned)key & 0xffffu;
                    lin = sLid[r[0]];
                } else if (P == 2) {
                    r[0] = ((unsigned)key >> 16) & 0xffffu;
                    r[1] = (unsigned)key & 0xffffu;
                    lin = (unsigned long long)sLid[r[0]] * g.k1k2 + sLid[R + r[1]];
                } else {
                    const uint32_t t12 = pt[((unsigned)key >> 16) & 0xffffu];
                    const uint32_t t34 = pt[L.npair + ((unsigned)key & 0xffffu)];
                    r[0] = t12 >> 16; r[1] = t12 & 0xffffu; r[2] = t34 >> 16; r[3] = t34 & 0xffffu;
                    lin = (unsigned long long)sLid[r[0]] * g.k1k2 + sLid[R + r[1]];
                    lin = lin * g.k1k2 + sLid[2 * R + r[2]];
                    lin = lin * g.k1k2 + sLid[3 * R + r[3]];
                }
                const unsigned long long slot = g.hashed ? (lin % g.H) : lin;
                const uint32_t o0 = g.offsets[slot], o1 = g.offsets[slot + 1];
                so0[t] = o0;
                slen[t] = o1 - o0;
                sslot[t] = (uint32_t)slot;
                if (g.tuples) {
                    uint16_t* tp = g.tuples + ((size_t)q * T + t) * 4;
                    tp[0] = (uint16_t)r[0]; tp[1] = (uint16_t)r[1]; tp[2] = (uint16_t)r[2]; tp[3] = (uint16_t)r[3];
                }
                if (g.tuple_keys) g.tuple_keys[(size_t)q * T + t] = mono_inv((uint32_t)(key >> 32));
                if (g.hashed) dkeys[t] = (slot << 32) | (unsigned)t;      // keys[t] is not needed again
            }
            if (g.n_tuples && tid == 0) g.n_tuples[q] = (uint32_t)Tn;
            __syncthreads();

            // ---- a slot proposed earlier in the order is skipped (hashed indexes only) --------------
            if (g.hashed) {
                const int Tpad = next_pow2(Tn);
                for (int e = Tn + tid; e < Tpad; e += kRankThreads) dkeys[e] = ~0ull;
                block_sort_lds(dkeys, Tpad, tid, kRankThreads);
                for (int e = tid + 1; e < Tn; e += kRankThreads) {
                    const unsigned long long cur = dkeys[e], prev = dkeys[e - 1];
                    if ((cur >> 32) == (prev >> 32)) slen[(unsigned)cur] = 0;   // not the first of its slot
                }
                __syncthreads();
            }

            // ---- lay the runs end to end, cut at C, compact --------------------------------------------
            // every thread takes `per` consecutive tuples; both prefix sums run in registers
            constexpr int kMaxPer = 8;                                      // Tn <= 8192 = kMaxPer * blockDim.x
            const int per = (Tn + kRankThreads - 1) / kRankThreads;
            const int t0 = tid * per;
            uint32_t len[kMaxPer], sum = 0;
#pragma unroll
            for (int i = 0; i < kMaxPer; ++i) {
                len[i] = (i < per && t0 + i < Tn) ? slen[t0 + i] : 0u;
                sum += len[i];
            }
            uint32_t total;
            uint32_t start = block_exclusive_sum(sum, part, total);
            if (attempt == 0 && total < C) continue;                        // not enough: rank all Tcap tuples
            uint32_t first[kMaxPer], flags = 0, nflag = 0;
#pragma unroll
            for (int i = 0; i < kMaxPer; ++i) {
                first[i] = start;
                if (len[i] > 0 && start < C) {                              // run is proposed
                    flags |= 1u << i;
                    ++nflag;
                }
                start += len[i];
            }
            uint32_t nruns;
            uint32_t idx = block_exclusive_sum(nflag, part + kRankThreads / kWave, nruns);
#pragma unroll
            for (int i = 0; i < kMaxPer; ++i) {
                if (((flags >> i) & 1u) == 0) continue;
                g.runs[(size_t)q * T + idx] = make_uint2(so0[t0 + i], first[i]);
                if (g.slots) g.slots[(size_t)q * T + idx] = sslot[t0 + i];
                ++idx;
            }
            if (tid == 0) g.meta[q] = make_uint2(nruns, total < C ? total : C);
            __syncthreads();
            break;
        }
    }   // next query of the list
}

hipError_t launch_rank(const RankArgs& a, hipStream_t s) {
    if (a.nq <= 0) return hipSuccess;
    const RankLds L = rank_layout(a.P, a.R, a.T, a.hashed);
    RankOffsets o;
    o.Tcap = L.Tcap; o.cap = L.cap; o.npair = L.npair; o.nreg = L.nreg; o.nreg_pair = L.nreg_pair;
    o.Tmid = L.Tmid; o.nreg_mid = L.nreg_mid;
    o.keys = (uint32_t)L.off_keys; o.hist = (uint32_t)L.off_hist;
    o.Ld = (uint32_t)L.off_Ld; o.Lid = (uint32_t)L.off_Lid; o.ps = (uint32_t)L.off_ps; o.pt = (uint32_t)L.off_pt;
    o.len = (uint32_t)L.off_len; o.o0 = (uint32_t)L.off_o0; o.slot = (uint32_t)L.off_slot;
    o.part = (uint32_t)L.off_part; o.misc = (uint32_t)L.off_misc;
    const bool taps = a.n_tuples || a.tuples || a.tuple_keys || a.slots;
    const bool head = (a.P == 2) && !taps;
    o.force = head ? 0 : 1;
    if (head) {
        constexpr int per = kRankHeadThreads / kWave;
        HeadLevels lv;
        lv.T1[0] = L.Tcap < kHeadT / 2 ? L.Tcap : kHeadT / 2;
        lv.T1[1] = L.Tcap < kHeadT ? L.Tcap : kHeadT;
        lv.npairs[0] = head_pair_count(lv.T1[0]);
        lv.npairs[1] = head_pair_count(lv.T1[1]);
        hipLaunchKernelGGL(rank_head_kernel, dim3((unsigned)((a.nq + per - 1) / per)), dim3(kRankHeadThreads), 0, s, a,
                           L.Tcap, lv);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const unsigned grid = head ? (unsigned)(a.nq < 1024 ? a.nq : 1024) : (unsigned)a.nq;
    hipLaunchKernelGGL(rank_kernel, dim3(grid), dim3(kRankThreads), L.total, s, a, o);
    return hipGetLastError();
}

hipError_t configure_rank(size_t max_dynamic_lds) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(rank_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
}

}  // namespace pqt
