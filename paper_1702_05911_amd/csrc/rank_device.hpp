// Device code of the full bin ranking of one query by one workgroup (any power-of-two size up to
// 1024 threads): used by the stand-alone ranking kernel and, for the few queries the head pass could
// not finish, inside the re-rank kernel.
#pragma once
#include "pqt_device.hpp"
#include "pqt_kernels.hpp"

namespace pqt {

__host__ __device__ inline int region_row_count(int a, int R, int T) {
    const int c = T / (a + 1);
    return c < R ? c : R;
}

constexpr int kSelBits = 10;
constexpr int kSelBins = 1 << kSelBits;
constexpr int kMidT = 128;         // tuples ranked first by the full pass; all T only if they do not fill C
constexpr int kRegionSplit = 64;   // rows below it are walked along b, the rest of the region along a
constexpr int kBinRankMax = 64;    // placing keys by histogram bin: most keys a bin may hold (each is ranked against its bin)
constexpr int kKeySlack = 64;      // entries of the key buffer beyond its power-of-two capacity (the last bin's excess)
constexpr int kPlaceBits = 11;
constexpr int kPlaceBins = 1 << kPlaceBits;    // bins of the placing histogram (the select path uses the first kSelBins)
constexpr int kPlaceMin = 256;     // regions up to this size are sorted as they are
constexpr int kRankPlace = 1;      // option of rank_pairs / rank_query

// Calls f(ordered sum bits, a, b) for every pair of the region {a < nA, b < nB, (a+1)(b+1) <= Tn},
// each pair once, spread over the workgroup.  Rows a < kRegionSplit are walked along b (they are
// long); the remaining pairs have b < Tn / (kRegionSplit + 1) and are walked along a, so lanes stay
// busy in the thin tail of the hyperbola as well.
// BOUNDED: only pairs whose key is at most `bound` are wanted (f is still called for a few others and
// tests the key itself): keys ascend along a row, so the wavefront leaves a row at the first 64 entries
// without a wanted key -- the first rows are many times longer than the part of them that matters, and
// without the bound most wavefronts would wait for the one that holds row 0.  (Dealing out units of 64
// entries instead of rows evens the walk as well, at a few instructions per unit; with the bound it gained
// nothing more: 0.765 against 0.766 ms per 10,000 queries on lists of 128.)
template <bool BOUNDED, typename F>
__device__ __forceinline__ void for_region(const float* A, int nA, const float* B, int nB, int Tn, int wave,
                                           int lane, uint32_t bound, F&& f) {
    const int nwaves = (int)blockDim.x / kWave;
    const int rows = min(min(nA, Tn), kRegionSplit);
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    // lane i holds the length of row i (and of column i below): one integer division per lane instead of one
    // per row, which was a fifth of the pass's instructions
    const int row_len = lane < rows ? region_row_count(lane, nB, Tn) : 0;
    for (int a = wv; a < rows; a += nwaves) {
        const int cnt = __builtin_amdgcn_readlane(row_len, a);
        const float da = A[a];
        for (int b = lane; b < cnt; b += kWave) {
            const uint32_t k32 = mono_key(da + B[b]);
            if (BOUNDED && __ballot(k32 <= bound) == 0) break;
            f(k32, (uint32_t)a, (uint32_t)b);
        }
    }
    if (nA > kRegionSplit) {
        const int cols = min(nB, Tn / (kRegionSplit + 1));
        const int col_end = (lane < cols && cols <= kWave) ? min(nA, Tn / (lane + 1)) : 0;
        for (int b = wv; b < cols; b += nwaves) {
            const int hi = cols <= kWave ? __builtin_amdgcn_readlane(col_end, b) : min(nA, Tn / (b + 1));
            const float db = B[b];
            for (int a = kRegionSplit + lane; a < hi; a += kWave) {
                const uint32_t k32 = mono_key(A[a] + db);
                if (BOUNDED && __ballot(k32 <= bound) == 0) break;
                f(k32, (uint32_t)a, (uint32_t)b);
            }
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
// Tn <= nA * nB; nreg = size of the region (a+1)(b+1) <= Tn; cap = a power of two >= Tn, keys[] holds
// cap entries (cap + kKeySlack where keys are placed by bin).  A small region is sorted as it is.
// Otherwise the keys are placed by counting: a 2048-bin histogram over the range that can hold the Tn-th
// key, a prefix sum that makes every bin's count its first position, a second walk that drops each key
// into its bin's range, and a last step in which every key counts the smaller keys of its own bin -- no
// comparison network.  Where a bin is too full for that (heavy ties) the Tn-th smallest key is found by
// a radix select over the region (sums recomputed in every pass, never stored), ties at that key are cut
// by (a, b), and only the Tn smallest are collected and sorted.  part: 16 words for the prefix sum.  All
// threads call it; ends with a barrier.
// MODE: kRankPlace = place by bin where possible (without it: the select-and-sort path only, which needs
// fewer registers where the ranking is a rarely taken branch of a larger kernel).
template <int MAXE, int MODE>
__device__ __forceinline__ void rank_pairs(const float* A, int nA, const float* B, int nB, int Tn, int nreg,
                                           int cap, unsigned long long* keys, uint32_t* hist, uint32_t* misc,
                                           uint32_t* part) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave, nt = blockDim.x;
    uint32_t tau = 0xffffffffu, a_cut = 0xffffffffu, b_cut = 0xffffffffu;
    const bool all = nreg <= (next_pow2(Tn) < 64 ? 64 : next_pow2(Tn));   // sorting the region costs no more than sorting Tn keys
    if ((MODE & kRankPlace) != 0 && nreg > kPlaceMin) {
        // ---- placing by bin -----------------------------------------------------------------------------
        // An upper bound of the Tn-th smallest key: the largest key of any rectangle a < sa, b < sb with
        // sa * sb >= Tn is its corner's (both lists ascend, rounding is monotone), and at least Tn keys are
        // not above it.  Lane l tries the rectangles with sa = l + 1 and with sb = l + 1 (lane 63: sa = nA, which
        // always qualifies because Tn <= nA * nB); the smallest corner bounds the histogram.
        const uint32_t lo_key = mono_key(A[0] + B[0]);
        uint32_t up_key;
        {
            const int s1 = lane == kWave - 1 ? nA : min(lane + 1, nA);
            const int o1 = (Tn + s1 - 1) / s1;
            up_key = o1 <= nB ? mono_key(A[s1 - 1] + B[o1 - 1]) : 0xffffffffu;
            const int s2 = min(lane + 1, nB);
            const int o2 = (Tn + s2 - 1) / s2;
            if (o2 <= nA) up_key = min(up_key, mono_key(A[o2 - 1] + B[s2 - 1]));
            up_key = wave_min_u32(up_key);
        }
        const uint32_t prange = up_key - lo_key;
        const int pwidth = 32 - __clz((int)(prange | 1u));
        const int pshift = pwidth > kPlaceBits ? pwidth - kPlaceBits : 0;
        for (int e = tid; e < kPlaceBins; e += nt) hist[e] = 0;
        if (tid == 0) misc[5] = 0;                       // a bin too full to rank, or more keys than keys[] holds
        __syncthreads();
        for_region<true>(A, nA, B, nB, Tn, wave, lane, up_key, [&](uint32_t k32, uint32_t, uint32_t) {
            if (k32 <= up_key) atomicAdd(&hist[(k32 - lo_key) >> pshift], 1u);
        });
        __syncthreads();
        {
            // counts -> first positions, in place; the thread that owns the bin of the Tn-th key notes it
            const int bpt = kPlaceBins / nt;             // bins per thread (nt a power of two, at most 1024)
            uint32_t sum = 0;
            for (int j = 0; j < bpt; ++j) sum += hist[tid * bpt + j];
            uint32_t total;
            uint32_t c = block_exclusive_sum(sum, part, total);
            for (int j = 0; j < bpt; ++j) {
                const uint32_t cnt = hist[tid * bpt + j];
                hist[tid * bpt + j] = c;
                if (c < (uint32_t)Tn) {
                    if (cnt > (uint32_t)kBinRankMax) misc[5] = 1;
                    if ((uint32_t)Tn <= c + cnt) {
                        misc[2] = (uint32_t)(tid * bpt + j);
                        misc[3] = c;
                        misc[4] = cnt;
                        if (c + cnt > (uint32_t)(cap + kKeySlack)) misc[5] = 1;
                    }
                }
                c += cnt;
            }
        }
        __syncthreads();
        if (misc[5] == 0) {
            const uint32_t bsel = misc[2], nkeys = misc[3] + misc[4];
            // the last key of bin bsel bounds this walk more tightly than the first one's bound
            const uint32_t last_key = min(up_key, lo_key + (((bsel + 1u) << pshift) - 1u));
            for_region<true>(A, nA, B, nB, Tn, wave, lane, last_key, [&](uint32_t k32, uint32_t a, uint32_t b) {
                if (k32 > last_key) return;
                keys[atomicAdd(&hist[(k32 - lo_key) >> pshift], 1u)] = ((unsigned long long)k32 << 32) | (a << 16) | b;
            });
            __syncthreads();
            // hist[b] is now the end of bin b (the start of bin b + 1) for every b <= bsel
            unsigned long long mine[MAXE + 1];
            uint32_t place[MAXE + 1];
#pragma unroll
            for (int i = 0; i < MAXE + 1; ++i) {
                const uint32_t e = (uint32_t)(tid + i * nt);
                place[i] = 0xffffffffu;
                if (e >= nkeys) continue;
                const unsigned long long key = keys[e];
                const uint32_t bin = ((uint32_t)(key >> 32) - lo_key) >> pshift;
                const uint32_t first = bin ? hist[bin - 1] : 0u, end = hist[bin];
                uint32_t r = first;
                for (uint32_t x = first; x < end; ++x) r += keys[x] < key ? 1u : 0u;
                mine[i] = key;
                place[i] = r;
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < MAXE + 1; ++i)
                if (place[i] < (uint32_t)Tn) keys[place[i]] = mine[i];
            __syncthreads();
            return;
        }
    }
    if (!all) {
        // ---- a bin was too full (or no placing): one histogram over the range of the region's keys ---
        const uint32_t lo_key = mono_key(A[0] + B[0]);
        // The region's smallest key is A[0]+B[0]; its largest is the last key of some row (both lists
        // ascend).  1024 bins over that range: the bin holding the Tn-th key is found, the
        // keys of lower bins go straight to keys[], the keys of that bin (a handful) to a side buffer
        // that reuses the histogram, is sorted, and gives its first Tn - (lower count).
        constexpr int kTailCap = kSelBins / 2;           // 64-bit entries the histogram's memory holds
        if (tid < 2) misc[tid] = 0;                      // [0] range maximum, [1] unused here
        for (int e = tid; e < kSelBins; e += nt) hist[e] = 0;
        __syncthreads();
        {
            const int rows = min(nA, Tn);               // every key of row a is <= the row's last key
            uint32_t kmax = lo_key;
            for (int a = tid; a < rows; a += nt)
                kmax = max(kmax, mono_key(A[a] + B[region_row_count(a, nB, Tn) - 1]));
            kmax = wave_max_u32(kmax);
            if (lane == 0 && kmax > lo_key) atomicMax(&misc[0], kmax);
        }
        __syncthreads();
        const uint32_t hi_key = max(misc[0], lo_key);
        const uint32_t range = hi_key - lo_key;
        const int width = 32 - __clz((int)(range | 1u));
        const int shift = width > kSelBits ? width - kSelBits : 0;
        for_region<false>(A, nA, B, nB, Tn, wave, lane, 0u, [&](uint32_t k32, uint32_t, uint32_t) {
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
            for_region<false>(A, nA, B, nB, Tn, wave, lane, 0u, [&](uint32_t k32, uint32_t a, uint32_t b) {
                const uint32_t bin = (k32 - lo_key) >> shift;
                const unsigned long long key = ((unsigned long long)k32 << 32) | (a << 16) | b;
                wave_append(bin < bsel, key, keys, &misc[0], lane);
                wave_append(bin == bsel, key, tail, &misc[1], lane);
            });
            __syncthreads();
            const int ntail = (int)inbin;
            const int tpad = next_pow2(ntail) < 64 ? 64 : next_pow2(ntail);
            for (int e = ntail + tid; e < tpad; e += nt) tail[e] = ~0ull;
            block_sort_lds<MAXE>(tail, tpad, tid, nt);
            for (int e = tid; e < Tn - (int)below; e += nt) keys[below + e] = tail[e];
            const int npad = next_pow2(Tn);
            for (int e = Tn + tid; e < npad; e += nt) keys[e] = ~0ull;
            block_sort_lds<MAXE>(keys, npad, tid, nt);
            return;
        }
        // ---- heavily tied keys: exact radix select ----------------------------------------------------
        __syncthreads();
        uint32_t prefix = 0, mask = 0, need = (uint32_t)Tn, less = 0, neq = 0;
        const int shifts[4] = {22, 12, 2, 0};
        const int nbits[4] = {10, 10, 10, 2};
        for (int pass = 0; pass < 4; ++pass) {
            for (int e = tid; e < kSelBins; e += nt) hist[e] = 0;
            __syncthreads();
            const int sh = shifts[pass];
            const uint32_t dm = (1u << nbits[pass]) - 1u;
            for_region<false>(A, nA, B, nB, Tn, wave, lane, 0u, [&](uint32_t k32, uint32_t, uint32_t) {
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
                for (int e = tid; e < kSelBins; e += nt) hist[e] = 0;
                __syncthreads();
                for_region<false>(A, nA, B, nB, Tn, wave, lane, 0u, [&](uint32_t k32, uint32_t a, uint32_t b) {
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
    for_region<false>(A, nA, B, nB, Tn, wave, lane, 0u, [&](uint32_t k32, uint32_t a, uint32_t b) {
        bool take = all || k32 < tau;
        if (!all && k32 == tau) take = a_cut == 0xffffffffu || a < a_cut || (a == a_cut && b <= b_cut);
        wave_append(take, ((unsigned long long)k32 << 32) | (a << 16) | b, keys, &misc[0], lane);
    });
    __syncthreads();
    const int n = (int)misc[0];
    const int npad = next_pow2(n);
    for (int e = n + tid; e < npad; e += nt) keys[e] = ~0ull;
    block_sort_lds<MAXE>(keys, npad, tid, nt);
}

// The full ranking of query q.  PF: 0 = the number of tree parts is read from g.P, 2 = it is two
// (the other cases are compiled out).  The run list goes to g.runs.  TO_LDS: (number of runs, number
// of candidates) go to out_counts[0..1] in LDS instead of g.meta (the caller goes on with the query).
// MAXPER (2, 4 or 8): tuples a thread may have to hold, L.Tcap <= MAXPER * blockDim.x.
// smem: the workgroup's LDS, laid out by L.  Every thread calls it; ends with a barrier.
template <int PF, bool TO_LDS, int MAXPER, int MODE>
__device__ __forceinline__ void rank_query(const RankArgs& g, const RankOffsets& L, int64_t q, unsigned char* smem,
                                           uint32_t* out_counts) {
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem + L.keys);
    unsigned long long* dkeys = keys;                       // (slot, position) keys reuse the sort buffer
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
    float* sLd = reinterpret_cast<float*>(smem + L.Ld);
    uint32_t* sLid = reinterpret_cast<uint32_t*>(smem + L.Lid);
    float* ps = reinterpret_cast<float*>(smem + L.ps);
    uint32_t* pt = reinterpret_cast<uint32_t*>(smem + L.pt);
    uint32_t* slen = reinterpret_cast<uint32_t*>(smem + L.len);
    uint32_t* sslot = reinterpret_cast<uint32_t*>(smem + L.slot);
    uint32_t* part = reinterpret_cast<uint32_t*>(smem + L.part);
    uint32_t* misc = reinterpret_cast<uint32_t*>(smem + L.misc);

    const int tid = threadIdx.x, nt = blockDim.x;
    const int P = PF ? PF : g.P, R = g.R, T = g.T;
    const uint32_t C = (uint32_t)g.C;

    for (int e = tid; e < P * R; e += nt) {
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
            for (int e = tid; e < Tn; e += nt)
                keys[e] = ((unsigned long long)mono_key(sLd[e]) << 32) | (unsigned)e;
            __syncthreads();                 // the list is already sorted by (distance, id)
        } else if (P == 2) {
            rank_pairs<MAXPER, MODE>(sLd, R, sLd + R, R, Tn, attempt == 0 ? L.nreg_mid : L.nreg, L.cap, keys, hist, misc,
                                     part);
        } else {
            // parts (1,2) and (3,4) first; then pairs of positions in those two lists.  One loop, so that the
            // ranking code exists once in the kernel: three copies of it do not fit the instruction cache.
            const int np = L.npair;
#pragma nounroll
            for (int stage = 0; stage < 3; ++stage) {
                const bool last = stage == 2;
                const float* A = last ? ps : sLd + 2 * stage * R;
                const float* B = last ? ps + np : sLd + (2 * stage + 1) * R;
                const int n = last ? np : R;
                rank_pairs<MAXPER, MODE>(A, n, B, n, last ? Tn : np, last ? L.nreg : L.nreg_pair, L.cap, keys, hist, misc,
                                         part);
                if (!last) {
                    for (int e = tid; e < np; e += nt) {
                        const unsigned long long key = keys[e];
                        ps[stage * np + e] = mono_inv((uint32_t)(key >> 32));
                        pt[stage * np + e] = (uint32_t)key;
                    }
                    __syncthreads();
                }
            }
        }

        // ---- tuple -> bin number -> slot -> run of the inverted list ---------------------------
        // every thread takes `per` consecutive tuples and keeps their runs in registers; LDS copies of the
        // run lengths and slots exist only where other threads need them (hashed slots, the slots tap)
        constexpr int kMaxPer = MAXPER;
        const int per = (Tn + nt - 1) / nt;
        const int t0 = tid * per;
        const bool keep_slots = g.hashed || g.slots;
        uint32_t len[kMaxPer], o0[kMaxPer];
#pragma unroll
        for (int i = 0; i < kMaxPer; ++i) {
            const int t = t0 + i;
            len[i] = 0;
            o0[i] = 0;
            if (i >= per || t >= Tn) continue;
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
            const unsigned long long slot = g.hashed ? slot_of_bin(lin, g.H, g.H_inv) : lin;
            o0[i] = g.offsets[slot];
            len[i] = g.offsets[slot + 1] - o0[i];
            if (keep_slots) sslot[t] = (uint32_t)slot;
            if (g.hashed) slen[t] = len[i];
            if (g.tuples) {
                uint16_t* tp = g.tuples + ((size_t)q * T + t) * 4;
                tp[0] = (uint16_t)r[0]; tp[1] = (uint16_t)r[1]; tp[2] = (uint16_t)r[2]; tp[3] = (uint16_t)r[3];
            }
            if (g.tuple_keys) g.tuple_keys[(size_t)q * T + t] = mono_inv((uint32_t)(key >> 32));
        }
        if (g.n_tuples && tid == 0) g.n_tuples[q] = (uint32_t)Tn;

        // ---- a slot proposed earlier in the order is skipped (hashed indexes only) --------------
        const int tsize = 2 * next_pow2(Tn);                  // at most half full; fits the keys' memory (2 * cap words)
        if (g.hashed && (MODE & kRankPlace) != 0 && tsize <= kPlaceBins) {
            // a table of (slot, first tuple) entries with open addressing in the memory of the histogram and
            // of the keys, both free by now: a tuple claims the entry of its slot (or finds it claimed for
            // the same slot), the smallest tuple number of an entry wins, the others' runs get length 0
            uint32_t* tslot = hist;
            uint32_t* tfirst = reinterpret_cast<uint32_t*>(keys);
            const int tshift = 32 - (31 - __clz(tsize));
            __syncthreads();                                  // every keys[t] has been read
            for (int e = tid; e < tsize; e += nt) {
                tslot[e] = 0xffffffffu;                       // no slot has this number: H < 2^32
                tfirst[e] = 0xffffffffu;
            }
            __syncthreads();
            uint32_t at[kMaxPer];
#pragma unroll
            for (int i = 0; i < kMaxPer; ++i) {
                const int t = t0 + i;
                at[i] = 0;
                if (i >= per || t >= Tn) continue;
                const uint32_t sl = sslot[t];
                uint32_t h = (sl * 2654435761u) >> tshift;
                for (;;) {
                    const uint32_t old = atomicCAS(&tslot[h], 0xffffffffu, sl);
                    if (old == 0xffffffffu || old == sl) break;
                    h = (h + 1) & (uint32_t)(tsize - 1);
                }
                atomicMin(&tfirst[h], (uint32_t)t);
                at[i] = h;
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < kMaxPer; ++i) {
                const int t = t0 + i;
                if (i < per && t < Tn && tfirst[at[i]] != (uint32_t)t) len[i] = 0;   // not the first of its slot
            }
        } else if (g.hashed) {
            __syncthreads();                                  // every keys[t] has been read
#pragma unroll
            for (int i = 0; i < kMaxPer; ++i) {
                const int t = t0 + i;
                if (i < per && t < Tn) dkeys[t] = ((unsigned long long)sslot[t] << 32) | (unsigned)t;
            }
            const int Tpad = next_pow2(Tn);
            for (int e = Tn + tid; e < Tpad; e += nt) dkeys[e] = ~0ull;
            block_sort_lds<MAXPER>(dkeys, Tpad, tid, nt);
            for (int e = tid + 1; e < Tn; e += nt) {
                const unsigned long long cur = dkeys[e], prev = dkeys[e - 1];
                if ((cur >> 32) == (prev >> 32)) slen[(unsigned)cur] = 0;   // not the first of its slot
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < kMaxPer; ++i)
                if (i < per && t0 + i < Tn) len[i] = slen[t0 + i];
        }

        // ---- lay the runs end to end, cut at C, compact --------------------------------------------
        uint32_t sum = 0;
#pragma unroll
        for (int i = 0; i < kMaxPer; ++i) sum += len[i];
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
        uint32_t idx = block_exclusive_sum(nflag, part + 16, nruns);
#pragma unroll
        for (int i = 0; i < kMaxPer; ++i) {
            if (((flags >> i) & 1u) == 0) continue;
            g.runs[(size_t)q * T + idx] = make_uint2(o0[i], first[i]);
            if (!TO_LDS && g.slots) g.slots[(size_t)q * T + idx] = sslot[t0 + i];
            ++idx;
        }
        if (tid == 0) {
            if (TO_LDS) {
                out_counts[0] = nruns;
                out_counts[1] = total < C ? total : C;
            } else {
                g.meta[q] = make_uint2(nruns, total < C ? total : C);
            }
        }
        __syncthreads();
        break;
    }
}

}  // namespace pqt
