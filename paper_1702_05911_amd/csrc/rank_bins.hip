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

int rank_region_size(int R, int T) {
    long n = 0;
    for (int a = 0; a < R; ++a) n += region_row_count(a, R, T);
    return (int)n;
}

constexpr int kSelBits = 10;
constexpr int kSelBins = 1 << kSelBits;

struct RankLds {
    int Tcap;   // tuples examined: min(T, R^P)
    int cap;    // sort buffer entries: next_pow2(Tcap)
    int nreg;   // size of the hyperbolic region (P = 2)
    size_t off_keys, off_dkeys, off_hist, off_Ld, off_Lid, off_rowbase, off_len, off_o0, off_flag, off_part,
        off_misc, total;
};

static RankLds rank_layout(int P, int R, int T, int hashed) {
    RankLds L;
    long total_tuples = 1;
    for (int p = 0; p < P; ++p) total_tuples = (total_tuples * R > (1L << 40)) ? (1L << 40) : total_tuples * R;
    L.Tcap = (int)((long)T < total_tuples ? (long)T : total_tuples);
    L.cap = next_pow2(L.Tcap) < 64 ? 64 : next_pow2(L.Tcap);
    L.nreg = (P == 1) ? L.Tcap : rank_region_size(R, L.Tcap);
    size_t o = 0;
    L.off_keys = o;    o += sizeof(unsigned long long) * L.cap;
    L.off_dkeys = o;   o += hashed ? sizeof(unsigned long long) * L.cap : 0;
    L.off_hist = o;    o += sizeof(uint32_t) * kSelBins;
    L.off_Ld = o;      o += sizeof(float) * P * R;
    L.off_Lid = o;     o += sizeof(uint32_t) * P * R;
    L.off_rowbase = o; o += sizeof(uint32_t) * (R + 1);
    L.off_len = o;     o += sizeof(uint32_t) * L.Tcap;
    L.off_o0 = o;      o += sizeof(uint32_t) * L.Tcap;
    L.off_flag = o;    o += sizeof(uint32_t) * L.Tcap;
    L.off_part = o;    o += sizeof(uint32_t) * (kRankThreads + 1);
    L.off_misc = o;    o += sizeof(uint32_t) * 16;
    L.total = o;
    return L;
}

size_t rank_lds_bytes(int P, int R, int T, int hashed) { return rank_layout(P, R, T, hashed).total; }

struct RankOffsets {   // layout handed to the kernel (computed once on the host)
    int Tcap, cap, nreg;
    int force;             // 1: rank every query (taps wanted, or no head pass ran)
    uint32_t keys, dkeys, hist, Ld, Lid, rowbase, len, o0, flag, part, misc;
};

constexpr int kHeadT = 64;                     // tuples the head pass ranks
constexpr int kHeadKeys = 320;                 // >= region size for R = T = 64 (280), in blocks of 64

// ------------------------------------------------------------------------------------------------
// Head pass.  Most queries reach the candidate budget C within the first few dozen tuples of the
// order (the later ones cannot change the result: their runs would start beyond C).  One wavefront
// per query ranks only the first min(T, 64) tuples exactly and, if their runs already fill C (or
// there are no more tuples), writes the final run list; otherwise it marks the query for the full
// pass.  Wave-synchronous: no workgroup barrier, LDS accesses of one wave execute in program order.
// ------------------------------------------------------------------------------------------------
struct HeadLds {
    float A[kHeadT], B[kHeadT];
    uint32_t Aid[kHeadT], Bid[kHeadT];
    unsigned long long keys[kHeadKeys];
    uint32_t slot[kHeadT];
};

#define PQT_WAVE_LDS_ORDER() wave_lds_order()

__device__ __forceinline__ void wave_compare_exchange(unsigned long long* keys, int i, int j, bool asc) {
    const unsigned long long x = keys[i], y = keys[j];
    if ((x > y) == asc) {
        keys[i] = y;
        keys[j] = x;
    }
}

__global__ __launch_bounds__(kRankThreads) void rank_head_kernel(RankArgs g, int Tn) {
    __shared__ HeadLds lds[kRankThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t q = (int64_t)blockIdx.x * (kRankThreads / kWave) + wave;
    if (q >= g.nq) return;
    HeadLds& S = lds[wave];
    const int R = g.R, T = g.T;
    const int R1 = R < kHeadT ? R : kHeadT;
    const int T1 = Tn < kHeadT ? Tn : kHeadT;

    if (lane < R1) {
        S.A[lane] = g.L_d[q * 2 * R + lane];
        S.Aid[lane] = g.L_id[q * 2 * R + lane];
        S.B[lane] = g.L_d[q * 2 * R + R + lane];
        S.Bid[lane] = g.L_id[q * 2 * R + R + lane];
    }
    PQT_WAVE_LDS_ORDER();

    // keys of the pairs with (r1+1)(r2+1) <= T1: lane = row r1
    const int cnt = (lane < R1) ? region_row_count(lane, R1, T1) : 0;
    const uint32_t incl = wave_inclusive_sum((uint32_t)cnt, lane);
    const int base = (int)incl - cnt;
    const int nreg = (int)__shfl(incl, kWave - 1, kWave);
    const int nblk = (nreg + kWave - 1) / kWave;
    {
        const float da = (lane < R1) ? S.A[lane] : 0.0f;
        for (int b = 0; b < cnt; ++b)
            S.keys[base + b] = ((unsigned long long)mono_key(da + S.B[b]) << 32) | ((unsigned)lane << 16) | (unsigned)b;
        for (int e = nreg + lane; e < nblk * kWave; e += kWave) S.keys[e] = ~0ull;
    }
    PQT_WAVE_LDS_ORDER();

    // sort every block of 64 keys ascending
    for (int size = 2; size <= kWave; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int c = lane; c < nblk * (kWave / 2); c += kWave) {
                const int blk = c / (kWave / 2), e = c % (kWave / 2);
                const int il = 2 * e - (e & (stride - 1));
                wave_compare_exchange(S.keys + blk * kWave, il, il + stride, (il & size) == 0);
            }
            PQT_WAVE_LDS_ORDER();
        }
    // fold the other blocks into block 0, keeping the 64 smallest each time: the lower half of the
    // union of two ascending runs is min(x[i], y[63-i]) (a bitonic sequence), then a bitonic merge
    for (int blk = 1; blk < nblk; ++blk) {
        const unsigned long long x = S.keys[lane], y = S.keys[blk * kWave + (kWave - 1 - lane)];
        S.keys[lane] = x < y ? x : y;
        PQT_WAVE_LDS_ORDER();
        for (int stride = kWave / 2; stride > 0; stride >>= 1) {
            if (lane < kWave / 2) {
                const int il = 2 * lane - (lane & (stride - 1));
                wave_compare_exchange(S.keys, il, il + stride, true);
            }
            PQT_WAVE_LDS_ORDER();
        }
    }

    // probe the first T1 tuples
    uint32_t o0 = 0, len = 0;
    if (lane < T1) {
        const unsigned long long key = S.keys[lane];
        const unsigned r1 = ((unsigned)key >> 16) & 0xffffu, r2 = (unsigned)key & 0xffffu;
        const unsigned long long lin = (unsigned long long)S.Aid[r1] * g.k1k2 + S.Bid[r2];
        const unsigned long long slot = g.hashed ? (lin % g.H) : lin;
        o0 = g.offsets[slot];
        len = g.offsets[slot + 1] - o0;
        S.slot[lane] = (uint32_t)slot;
    }
    if (g.hashed) {
        PQT_WAVE_LDS_ORDER();
        if (lane < T1) {
            const uint32_t mine = S.slot[lane];
            for (int t = 0; t < lane; ++t)
                if (S.slot[t] == mine) len = 0;          // proposed earlier in the order
        }
    }
    const uint32_t incl_len = wave_inclusive_sum(len, lane);
    const uint32_t start = incl_len - len;
    const uint32_t total = __shfl(incl_len, kWave - 1, kWave);
    const uint32_t C = (uint32_t)g.C;
    if (total < C && T1 < Tn) {                          // not enough yet and more tuples exist
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
}

// ------------------------------------------------------------------------------------------------
// Full pass: workgroups take the queries the head pass listed (or every query when forced).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kRankThreads) void rank_kernel(RankArgs g, RankOffsets L) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem + L.keys);
    unsigned long long* dkeys = reinterpret_cast<unsigned long long*>(smem + L.dkeys);
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
    float* sLd = reinterpret_cast<float*>(smem + L.Ld);
    uint32_t* sLid = reinterpret_cast<uint32_t*>(smem + L.Lid);
    uint32_t* rowbase = reinterpret_cast<uint32_t*>(smem + L.rowbase);
    uint32_t* slen = reinterpret_cast<uint32_t*>(smem + L.len);
    uint32_t* so0 = reinterpret_cast<uint32_t*>(smem + L.o0);
    uint32_t* sflag = reinterpret_cast<uint32_t*>(smem + L.flag);
    uint32_t* part = reinterpret_cast<uint32_t*>(smem + L.part);
    uint32_t* misc = reinterpret_cast<uint32_t*>(smem + L.misc);

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    constexpr int nwaves = kRankThreads / kWave;
    const int P = g.P, R = g.R, T = g.T;
    const int Tn = L.Tcap;                                  // min(T, R^P)
    const uint32_t C = (uint32_t)g.C;
    const uint32_t count = L.force ? (uint32_t)g.nq : g.todo[0];
    for (uint32_t item = blockIdx.x; item < count; item += gridDim.x) {
        const int64_t q = L.force ? (int64_t)item : (int64_t)g.todo[1 + item];

        for (int e = tid; e < P * R; e += kRankThreads) {
            sLd[e] = g.L_d[q * P * R + e];
            sLid[e] = g.L_id[q * P * R + e];
        }
        __syncthreads();

        // ---- the first Tn tuples, sorted, as keys (ordered sum bits, r1, r2) -----------------------
        if (P == 1) {
            for (int e = tid; e < Tn; e += kRankThreads)
                keys[e] = ((unsigned long long)mono_key(sLd[e]) << 32) | (unsigned)e;
            __syncthreads();                     // the list is already sorted by (distance, id)
        } else if (L.nreg <= L.cap) {            // the whole region fits: sort it
            for (int a = tid; a < R; a += kRankThreads) rowbase[a] = (uint32_t)region_row_count(a, R, Tn);
            __syncthreads();
            const uint32_t nreg = block_exclusive_scan(rowbase, R, part);
            const int npad = next_pow2((int)nreg);
            for (int a = wave; a < R; a += nwaves) {
                const int cnt = region_row_count(a, R, Tn);
                const uint32_t base = rowbase[a];
                const float da = sLd[a];
                for (int b = lane; b < cnt; b += kWave)
                    keys[base + b] = ((unsigned long long)mono_key(da + sLd[R + b]) << 32) | ((unsigned)a << 16) | (unsigned)b;
            }
            for (int e = (int)nreg + tid; e < npad; e += kRankThreads) keys[e] = ~0ull;
            bitonic_sort_lds(keys, npad, tid, kRankThreads);
        } else {
            // radix select of the Tn-th smallest sum over the region, keys recomputed in every pass
            const int rows = R < Tn ? R : Tn;
            auto for_region = [&](auto&& f) {
                for (int a = wave; a < rows; a += nwaves) {
                    const int cnt = region_row_count(a, R, Tn);
                    const float da = sLd[a];
                    for (int b = lane; b < cnt; b += kWave) f(mono_key(da + sLd[R + b]), (uint32_t)a, (uint32_t)b);
                }
            };
            uint32_t prefix = 0, mask = 0, need = (uint32_t)Tn, less = 0, neq = 0;
            const int shifts[4] = {22, 12, 2, 0};
            const int nbits[4] = {10, 10, 10, 2};
            for (int pass = 0; pass < 4; ++pass) {
                for (int e = tid; e < kSelBins; e += kRankThreads) hist[e] = 0;
                __syncthreads();
                const int sh = shifts[pass];
                const uint32_t dm = (1u << nbits[pass]) - 1u;
                for_region([&](uint32_t k32, uint32_t, uint32_t) {
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
            const uint32_t tau = prefix;                     // Tn-th smallest sum key; `need` of the neq ties count
            uint32_t a_cut = 0xffffffffu, b_cut = 0xffffffffu;
            if (less + neq > (uint32_t)L.cap) {              // too many ties: cut them by (r1, r2)
                for (int e = tid; e < kSelBins; e += kRankThreads) hist[e] = 0;
                __syncthreads();
                for_region([&](uint32_t k32, uint32_t a, uint32_t) {
                    if (k32 == tau) atomicAdd(&hist[a], 1u);
                });
                __syncthreads();
                uint32_t before, cnt;
                hist_locate(hist, need, lane, a_cut, before, cnt);
                need -= before;
                __syncthreads();
                for (int e = tid; e < kSelBins; e += kRankThreads) hist[e] = 0;
                __syncthreads();
                for_region([&](uint32_t k32, uint32_t a, uint32_t b) {
                    if (k32 == tau && a == a_cut) atomicAdd(&hist[b], 1u);
                });
                __syncthreads();
                hist_locate(hist, need, lane, b_cut, before, cnt);
                __syncthreads();
            }
            if (tid == 0) misc[0] = 0;
            __syncthreads();
            for_region([&](uint32_t k32, uint32_t a, uint32_t b) {
                bool take = k32 < tau;
                if (k32 == tau) take = a_cut == 0xffffffffu || a < a_cut || (a == a_cut && b <= b_cut);
                if (take) keys[atomicAdd(&misc[0], 1u)] = ((unsigned long long)k32 << 32) | (a << 16) | b;
            });
            __syncthreads();
            const int n = (int)misc[0];
            const int npad = next_pow2(n);
            for (int e = n + tid; e < npad; e += kRankThreads) keys[e] = ~0ull;
            bitonic_sort_lds(keys, npad, tid, kRankThreads);
        }

        // ---- tuple -> bin number -> slot -> run of the inverted list -------------------------------
        for (int t = tid; t < Tn; t += kRankThreads) {
            const unsigned long long key = keys[t];
            unsigned long long lin;
            unsigned r1, r2 = 0;
            if (P == 1) {
                r1 = (unsigned)key & 0xffffu;
                lin = sLid[r1];
            } else {
                r1 = ((unsigned)key >> 16) & 0xffffu;
                r2 = (unsigned)key & 0xffffu;
                lin = (unsigned long long)sLid[r1] * g.k1k2 + sLid[R + r2];
            }
            const unsigned long long slot = g.hashed ? (lin % g.H) : lin;
            const uint32_t o0 = g.offsets[slot], o1 = g.offsets[slot + 1];
            so0[t] = o0;
            slen[t] = o1 - o0;
            if (g.hashed) dkeys[t] = (slot << 32) | (unsigned)t;
            if (g.tuples) {
                uint16_t* tp = g.tuples + ((size_t)q * T + t) * 4;
                tp[0] = (uint16_t)r1; tp[1] = (uint16_t)r2; tp[2] = 0; tp[3] = 0;
            }
            if (g.tuple_keys) g.tuple_keys[(size_t)q * T + t] = mono_inv((uint32_t)(key >> 32));
        }
        if (g.n_tuples && tid == 0) g.n_tuples[q] = (uint32_t)Tn;
        __syncthreads();

        // ---- a slot proposed earlier in the order is skipped (hashed indexes only) ------------------
        if (g.hashed) {
            const int Tpad = next_pow2(Tn);
            for (int e = Tn + tid; e < Tpad; e += kRankThreads) dkeys[e] = ~0ull;
            bitonic_sort_lds(dkeys, Tpad, tid, kRankThreads);
            for (int e = tid + 1; e < Tn; e += kRankThreads) {
                const unsigned long long cur = dkeys[e], prev = dkeys[e - 1];
                if ((cur >> 32) == (prev >> 32)) slen[(unsigned)cur] = 0;   // not the first of its slot
            }
            __syncthreads();
        }

        // ---- lay the runs end to end, cut at C, compact ------------------------------------------------
        for (int t = tid; t < Tn; t += kRankThreads) sflag[t] = slen[t];
        __syncthreads();
        const uint32_t total = block_exclusive_scan(sflag, Tn, part);    // sflag[t] = start position
        for (int t = tid; t < Tn; t += kRankThreads) {
            const uint32_t start = sflag[t];
            slen[t] = (slen[t] > 0 && start < C) ? 1u : 0u;              // run is proposed
        }
        __syncthreads();
        const uint32_t nruns = block_exclusive_scan(slen, Tn, part);    // slen[t] = run index
        for (int t = tid; t < Tn; t += kRankThreads) {
            const uint32_t start = sflag[t];
            const uint32_t idx = slen[t];
            const bool emit = (t + 1 < Tn ? slen[t + 1] : nruns) != idx; // its flag was 1
            if (emit) {
                g.runs[(size_t)q * T + idx] = make_uint2(so0[t], start);
                if (g.slots) {
                    const unsigned long long key = keys[t];
                    unsigned long long lin;
                    if (P == 1) lin = sLid[(unsigned)key & 0xffffu];
                    else lin = (unsigned long long)sLid[((unsigned)key >> 16) & 0xffffu] * g.k1k2 + sLid[R + ((unsigned)key & 0xffffu)];
                    g.slots[(size_t)q * T + idx] = g.hashed ? (lin % g.H) : lin;
                }
            }
        }
        if (tid == 0) g.meta[q] = make_uint2(nruns, total < C ? total : C);
        __syncthreads();
    }   // next query of the list
}

hipError_t launch_rank(const RankArgs& a, hipStream_t s) {
    if (a.nq <= 0) return hipSuccess;
    const RankLds L = rank_layout(a.P, a.R, a.T, a.hashed);
    RankOffsets o;
    o.Tcap = L.Tcap; o.cap = L.cap; o.nreg = L.nreg;
    o.keys = (uint32_t)L.off_keys; o.dkeys = (uint32_t)L.off_dkeys; o.hist = (uint32_t)L.off_hist;
    o.Ld = (uint32_t)L.off_Ld; o.Lid = (uint32_t)L.off_Lid; o.rowbase = (uint32_t)L.off_rowbase;
    o.len = (uint32_t)L.off_len; o.o0 = (uint32_t)L.off_o0; o.flag = (uint32_t)L.off_flag;
    o.part = (uint32_t)L.off_part; o.misc = (uint32_t)L.off_misc;
    const bool taps = a.n_tuples || a.tuples || a.tuple_keys || a.slots;
    const bool head = (a.P == 2) && !taps;
    o.force = head ? 0 : 1;
    if (head) {
        constexpr int per = kRankThreads / kWave;
        hipLaunchKernelGGL(rank_head_kernel, dim3((unsigned)((a.nq + per - 1) / per)), dim3(kRankThreads), 0, s, a,
                           L.Tcap);
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
