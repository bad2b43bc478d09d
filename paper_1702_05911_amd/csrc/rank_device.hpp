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

// Calls f(ordered sum bits, a, b) for every pair of the region {a < nA, b < nB, (a+1)(b+1) <= Tn},
// each pair once, spread over the workgroup.  Rows a < kRegionSplit are walked along b (they are
// long); the remaining pairs have b < Tn / (kRegionSplit + 1) and are walked along a, so lanes stay
// busy in the thin tail of the hyperbola as well.
template <typename F>
__device__ __forceinline__ void for_region(const float* A, int nA, const float* B, int nB, int Tn, int wave,
                                           int lane, F&& f) {
    const int nwaves = (int)blockDim.x / kWave;
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
template <int MAXE>
__device__ __forceinline__ void rank_pairs(const float* A, int nA, const float* B, int nB, int Tn, int nreg,
                                           int cap, unsigned long long* keys, uint32_t* hist, uint32_t* misc) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave, nt = blockDim.x;
    uint32_t tau = 0xffffffffu, a_cut = 0xffffffffu, b_cut = 0xffffffffu;
    const bool all = nreg <= (next_pow2(Tn) < 64 ? 64 : next_pow2(Tn));   // sorting the region costs no more than sorting Tn keys
    if (!all) {
        // ---- usual case: one histogram over the range of the region's keys ----------------------------
        // The region's smallest key is A[0]+B[0]; its largest is the last key of some row (both lists
        // ascend).  1024 bins over that range: the bin holding the Tn-th key is found, the
        // keys of lower bins go straight to keys[], the keys of that bin (a handful) to a side buffer
        // that reuses the histogram, is sorted, and gives its first Tn - (lower count).
        constexpr int kTailCap = kSelBins / 2;           // 64-bit entries the histogram's memory holds
        const uint32_t lo_key = mono_key(A[0] + B[0]);
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
                for (int e = tid; e < kSelBins; e += nt) hist[e] = 0;
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
    for (int e = n + tid; e < npad; e += nt) keys[e] = ~0ull;
    block_sort_lds<MAXE>(keys, npad, tid, nt);
}

// The full ranking of query q.  PF: 0 = the number of tree parts is read from g.P, 2 = it is two
// (the other cases are compiled out).  The run list goes to g.runs.  TO_LDS: (number of runs, number
// of candidates) go to out_counts[0..1] in LDS instead of g.meta (the caller goes on with the query).
// MAXPER (2, 4 or 8): tuples a thread may have to hold, L.Tcap <= MAXPER * blockDim.x.
// smem: the workgroup's LDS, laid out by L.  Every thread calls it; ends with a barrier.
template <int PF, bool TO_LDS, int MAXPER>
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
            rank_pairs<MAXPER>(sLd, R, sLd + R, R, Tn, attempt == 0 ? L.nreg_mid : L.nreg, L.cap, keys, hist, misc);
        } else {
            // parts (1,2) and (3,4) first; then pairs of positions in those two lists
            const int np = L.npair;
            for (int half = 0; half < 2; ++half) {
                rank_pairs<MAXPER>(sLd + 2 * half * R, R, sLd + (2 * half + 1) * R, R, np, L.nreg_pair, L.cap, keys, hist,
                           misc);
                for (int e = tid; e < np; e += nt) {
                    const unsigned long long key = keys[e];
                    ps[half * np + e] = mono_inv((uint32_t)(key >> 32));
                    pt[half * np + e] = (uint32_t)key;
                }
                __syncthreads();
            }
            rank_pairs<MAXPER>(ps, np, ps + np, np, Tn, L.nreg, L.cap, keys, hist, misc);
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
            const unsigned long long slot = g.hashed ? (lin % g.H) : lin;
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
        if (g.hashed) {
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
