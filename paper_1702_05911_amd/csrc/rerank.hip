// Vector proposal, re-ranking by line quantisation and the final ordering
// (Sec. 3.2 "vector proposal", Sec. 3.3 "Online computation" Eq. 8-9, Sec. 4 last kernel).
//
// One workgroup per query.
//   * the per-query table LUT[m][c] of Eq. 9 summands is built in LDS from the level-1
//     sub-part distances the traversal already produced (no new distance is computed);
//   * codes are stored bin-major beside the ids, so the candidates of a proposed slot are one
//     contiguous run: a thread's candidate positions only grow, so it walks the run starts (in
//     LDS) forwards; consecutive lanes read consecutive codes (coalesced), eight positions per
//     thread in flight; the id array is only touched for the few survivors;
//   * score = sum over m = 0..M-1, in that order, of LUT[m][code[m]] in fp32;
//   * the k best by (score, id): one 1024-bin histogram over the ordered score bits between the
//     smallest and largest score of the query; every wavefront locates the bin b that holds the
//     k-th smallest; the positions in bins <= b (a superset of the answer, normally a few more
//     than k) are compacted, their ids fetched, and the (score bits, id) keys ordered by counting
//     ranks, four lanes per survivor.  If the superset does not fit (heavily tied scores) an
//     exact radix select on score bits, then on ids, picks exactly k.
#include "rank_device.hpp"

namespace pqt {

constexpr int kHistBits = 10;
constexpr int kHistSize = 1 << kHistBits;
constexpr int kCountRankMax = 512;   // survivors ordered by counting ranks up to this many, else bitonic
constexpr int kRunPrefetch = 64;     // runs fetched before the run count is known
constexpr int kFusedPer = 2;         // tuples per thread the in-kernel bin ranking may hold (keeps registers low)

struct RerankLds {
    int kpad, scap;
    uint32_t surv, spos, lut, a, run_src, run_start, skey, hist, misc, total;
};

// (pair, lambda) codes: entries per sub-part in the LDS table of centroid pairs (128 while the pairs fit)
static int pair_table_shift(int k1) { return k1 * (k1 - 1) / 2 <= 128 ? 7 : 8; }

static RerankLds rerank_layout(int M, int k1, int T, int C, int k, int threads, size_t rank_lds, int code_format) {
    RerankLds L;
    (void)threads;
    L.kpad = next_pow2(k);
    L.scap = 2 * L.kpad < 256 ? 256 : 2 * L.kpad;
    size_t o = 0;
    // at offset 0: lookups need no base register; also the scan scratch of the exact fallback.
    // One float per table entry, or (b^2, a^2 - b^2, c^2, -) per centroid pair for (pair, lambda) codes.
    L.lut = (uint32_t)o;       o += code_format == 1 ? sizeof(float4) * ((size_t)M << pair_table_shift(k1)) : sizeof(float) * M * 256;
    L.skey = (uint32_t)o;      o += sizeof(uint32_t) * ((C + 3) & ~3);
    L.surv = (uint32_t)o;      o += sizeof(unsigned long long) * L.scap;
    L.hist = (uint32_t)o;      o += sizeof(uint32_t) * kHistSize;
    // everything above is free while a workgroup runs the full bin ranking of its query, which uses
    // the first rank_lds bytes; the arrays below receive its result
    if (o < rank_lds) o = (rank_lds + 15) & ~size_t(15);
    L.a = (uint32_t)o;         o += sizeof(float) * M * k1;
    L.run_src = (uint32_t)o;   o += sizeof(uint32_t) * T;
    L.run_start = (uint32_t)o; o += sizeof(uint32_t) * (T + 1);
    L.misc = (uint32_t)o;      o += sizeof(uint32_t) * 16;
    L.spos = (uint32_t)o;      o += sizeof(uint16_t) * L.scap;
    o = (o + 15) & ~size_t(15);
    L.total = (uint32_t)o;
    return L;
}

size_t rerank_lds_bytes(int M, int k1, int T, int C, int k, int threads, size_t rank_lds, int code_format) {
    return rerank_layout(M, k1, T, C, k, threads, rank_lds, code_format).total;
}

// Position p of the candidate list -> position in ids/codes: the run r with
// run_start[r] <= p < run_start[r+1], found in `steps` = ceil(log2(nr)) halvings.
__device__ __forceinline__ uint32_t source_of(uint32_t p, int nr, int steps, const uint32_t* run_src,
                                              const uint32_t* run_start) {
    int lo = 0, hi = nr;
    for (int s = 0; s < steps; ++s) {
        const int mid = (lo + hi) >> 1;
        const bool ge = run_start[mid] <= p;
        lo = ge ? mid : lo;
        hi = ge ? hi : mid;
    }
    return run_src[lo] + (p - run_start[lo]);
}

// One pass of a most-significant-digit radix select (exact fallback).  Counts, among the n items
// whose key agrees with `prefix` on the bits of `mask`, the digit (key >> shift) & (2^bits - 1);
// finds the digit holding the item of 1-based rank `need`.  out[0] = digit, out[1] = rank inside
// it, out[2] = size of the chosen digit's bucket.  All threads must call it; ends with a barrier.
template <typename KeyFn>
__device__ __forceinline__ void radix_select_pass(int n, uint32_t prefix, uint32_t mask, int shift, int bits,
                                                  uint32_t need, uint32_t* hist, uint32_t* part,
                                                  uint32_t* out, KeyFn get_key) {
    const int tid = threadIdx.x, nt = blockDim.x;
    const int nb = 1 << bits;
    for (int e = tid; e < nb; e += nt) hist[e] = 0;
    __syncthreads();
    for (int p = tid; p < n; p += nt) {
        bool valid;
        const uint32_t key = get_key(p, valid);
        if (valid && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
    }
    __syncthreads();
    const int chunk = (nb + nt - 1) / nt;
    const int lo = min(tid * chunk, nb), hi = min(lo + chunk, nb);
    uint32_t s = 0;
    for (int e = lo; e < hi; ++e) s += hist[e];
    part[tid] = s;
    __syncthreads();
    for (int off = 1; off < nt; off <<= 1) {
        uint32_t v = (tid >= off) ? part[tid - off] : 0u;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    s = (tid > 0) ? part[tid - 1] : 0u;
    for (int e = lo; e < hi; ++e) {
        const uint32_t c = hist[e];
        if (s < need && need <= s + c) {
            out[0] = (uint32_t)e;
            out[1] = need - s;
            out[2] = c;
        }
        s += c;
    }
    __syncthreads();
}

// misc words
enum { kMin = 0, kMax = 1, kSel = 2, kSelCount = 3, kNumSurv = 4, kRadix = 8, kRanked = 12 };

// LUT[m][c] read through an LDS address formed from the code byte alone: the table sits at LDS
// address 0 (the kernels here have no static LDS; the launcher checks that), so the address is
// c * 4 plus the compile-time offset m * 1024 -- one sub-dword shift per lookup.
typedef __attribute__((address_space(3))) const float lds_cfloat;
__device__ __forceinline__ float lut_at(int m, uint32_t c) {
    return *reinterpret_cast<lds_cfloat*>((uintptr_t)((c << 2) + (uint32_t)m * 1024u));
}

// The run a thread's current candidate position lies in, kept in registers: positions of a thread
// only grow, so the run only moves forwards and LDS is read only when a position crosses into the
// next run.
struct RunCursor {
    int run;
    uint32_t next_start;   // run_start[run + 1]
    uint32_t delta;        // run_src[run] - run_start[run]: position in ids/codes = candidate position + delta
};

// (pair, lambda level) codes: the summand of Eq. 9 for one sub-part from the pair's LDS entry
// (b^2, a^2 - b^2, c^2) and the level; lambda = (level - 96) / 16 is exact in fp32.
constexpr int kPairLambda = -1;      // MW < 0 selects this code format: -1 any M (byte loads), else -(words per code)
__device__ __forceinline__ float pair_lambda_term(const float4* plut, int shift, int m, uint32_t pair, uint32_t level) {
    const float4 e = plut[(m << shift) + pair];
    const float lam = fmaf((float)level, 0.0625f, -6.0f);
    return fmaf(fmaf(lam, lam, -lam), e.z, fmaf(lam, e.y, e.x));
}

// Scores U candidate positions per thread (base + u*nt + tid).  CHECK: positions may pass nc.
template <int MW, int U, bool CHECK, bool TAPS>
__device__ __forceinline__ void score_batch(const RerankArgs& g, int64_t q, int base, int nc, int tid, int nt,
                                            const float* lut, uint32_t* skey, const uint32_t* run_src,
                                            const uint32_t* run_start, RunCursor& cur, uint32_t& kmin,
                                            uint32_t& kmax) {
    constexpr int NW = MW > 0 ? MW : (MW < -1 ? -MW : 0);      // code words fetched up front (0: byte loads)
    const int M = MW > 0 ? 4 * MW : (MW < -1 ? -2 * MW : g.M);
    uint32_t src[U];
    uint32_t cw[U][NW > 0 ? NW : 1];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t p = (uint32_t)(base + u * nt + tid);
        if (!CHECK || p < (uint32_t)nc) {
            while (p >= cur.next_start) {                          // run_start[nr] = nc > p ends the walk
                ++cur.run;
                cur.next_start = run_start[cur.run + 1];
                cur.delta = run_src[cur.run] - run_start[cur.run];
            }
            src[u] = p + cur.delta;
        } else {
            src[u] = run_src[0];
        }
    }
    if (NW > 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t* c = reinterpret_cast<const uint32_t*>(g.codes + (size_t)src[u] * (4 * NW));
            if (NW == 2) {
                const uint2 v = *reinterpret_cast<const uint2*>(c);
                cw[u][0] = v.x;
                cw[u][NW > 1 ? 1 : 0] = v.y;
            } else if (NW == 4) {
                const uint4 v = *reinterpret_cast<const uint4*>(c);
                cw[u][0] = v.x;
                cw[u][NW > 1 ? 1 : 0] = v.y;
                cw[u][NW > 2 ? 2 : 0] = v.z;
                cw[u][NW > 3 ? 3 : 0] = v.w;
            } else {
#pragma unroll
                for (int j = 0; j < NW; ++j) cw[u][j] = c[j];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int p = base + u * nt + tid;
        if (CHECK && p >= nc) continue;
        float s;
        if (MW > 0) {
            s = lut_at(0, cw[u][0] & 0xffu);               // sum in ascending m
            s += lut_at(1, (cw[u][0] >> 8) & 0xffu);
            s += lut_at(2, (cw[u][0] >> 16) & 0xffu);
            s += lut_at(3, cw[u][0] >> 24);
#pragma unroll
            for (int j = 1; j < MW; ++j) {
                const uint32_t wv = cw[u][j];
                s += lut_at(j * 4 + 0, wv & 0xffu);
                s += lut_at(j * 4 + 1, (wv >> 8) & 0xffu);
                s += lut_at(j * 4 + 2, (wv >> 16) & 0xffu);
                s += lut_at(j * 4 + 3, wv >> 24);
            }
        } else if (MW < -1) {
            // two bytes per sub-part, two sub-parts per word
            const float4* plut = reinterpret_cast<const float4*>(lut);
            s = 0.0f;
#pragma unroll
            for (int j = 0; j < NW; ++j) {
                const uint32_t wv = cw[u][j];
                s += pair_lambda_term(plut, g.pair_shift, 2 * j, wv & 0xffu, (wv >> 8) & 0xffu);
                s += pair_lambda_term(plut, g.pair_shift, 2 * j + 1, (wv >> 16) & 0xffu, wv >> 24);
            }
        } else if (MW == kPairLambda) {
            const float4* plut = reinterpret_cast<const float4*>(lut);
            const uint8_t* code = g.codes + (size_t)src[u] * 2 * M;
            s = 0.0f;
            for (int m = 0; m < M; ++m) s += pair_lambda_term(plut, g.pair_shift, m, code[2 * m], code[2 * m + 1]);
        } else {
            const uint8_t* code = g.codes + (size_t)src[u] * M;
            s = 0.0f;
            for (int m = 0; m < M; ++m) s += lut[m * 256 + code[m]];
        }
        const uint32_t key = mono_key(s);
        skey[p] = key;
        kmin = min(kmin, key);
        kmax = max(kmax, key);
        if (TAPS) {
            if (g.scores) g.scores[(size_t)q * g.C + p] = s;
            if (g.cand_ids) g.cand_ids[(size_t)q * g.C + p] = (int64_t)g.ids[src[u]];
        }
    }
}

// MW = 32-bit words per code (M/4) for M in {4, 8, 16, 32}; 0 = any other M (byte loads);
// kPairLambda = codes hold (centroid pair, lambda level) per sub-part, scored by Eq. 9 directly.
// FUSED: a query whose meta.x is kMetaTodo (the ranking head pass could not finish it) is first
// ranked in full by this workgroup, which leaves the run list directly in LDS.
template <int MW, bool TAPS, bool FUSED>
__global__ __launch_bounds__(1024, FUSED ? 8 : 1) void rerank_kernel(RerankArgs g, RerankLds L, RankArgs rk, RankOffsets RL) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* surv = reinterpret_cast<unsigned long long*>(smem + L.surv);
    uint16_t* spos = reinterpret_cast<uint16_t*>(smem + L.spos);
    float* lut = reinterpret_cast<float*>(smem);                 // L.lut == 0
    float* sa = reinterpret_cast<float*>(smem + L.a);
    uint32_t* run_src = reinterpret_cast<uint32_t*>(smem + L.run_src);
    uint32_t* run_start = reinterpret_cast<uint32_t*>(smem + L.run_start);
    uint32_t* skey = reinterpret_cast<uint32_t*>(smem + L.skey);
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
    uint32_t* misc = reinterpret_cast<uint32_t*>(smem + L.misc);

    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int M = g.M, k1 = g.k1, T = g.T, k = g.k;
    const int nlut = M * 256;

    int64_t q;
    uint2 meta;
    if ((int)blockIdx.x < g.early) {           // one of the queries the head pass left unfinished, if any
        if (blockIdx.x >= *g.todo_count) return;
        q = (int64_t)g.todo[blockIdx.x];
        meta = g.meta[q];
    } else {
        q = (int64_t)blockIdx.x - g.early;
        meta = g.meta[q];
        if (g.early > 0 && meta.x == kMetaTodo && meta.y < (uint32_t)g.early) return;   // an early workgroup has it
    }
    bool ranked_here = false;
    if (FUSED && meta.x == kMetaTodo) {        // same for the whole workgroup
        rank_query<2, true, kFusedPer>(rk, RL, q, smem, run_src, run_start, misc + kRanked);
        meta = make_uint2(misc[kRanked], misc[kRanked + 1]);
        ranked_here = true;
    }

    // ---- issue every load that needs no other result first ------------------------------------------
    uint2 run0 = make_uint2(0u, 0u);
    if (!ranked_here && tid < kRunPrefetch && tid < T) run0 = g.runs[(size_t)q * T + tid];
    CodeEntry ent[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int e = u * nt + tid;
        ent[u] = g.table[e < nlut ? e : 0];
    }
    for (int e = tid; e < M * k1; e += nt) sa[e] = g.a[(size_t)q * M * k1 + e];
    for (int e = tid; e < kHistSize; e += nt) hist[e] = 0;
    const int nr = (int)meta.x;
    const int nc = (int)meta.y;
    int steps = 0;
    while ((1 << steps) < nr) ++steps;
    if (!ranked_here) {
        if (tid < kRunPrefetch && tid < nr) {
            run_src[tid] = run0.x;
            run_start[tid] = run0.y;
        }
        for (int r = kRunPrefetch + tid; r < nr; r += nt) {
            const uint2 run = g.runs[(size_t)q * T + r];
            run_src[r] = run.x;
            run_start[r] = run.y;
        }
    }
    if (tid == 0) {
        run_start[nr] = (uint32_t)nc;
        misc[kMin] = 0xffffffffu;
        misc[kMax] = 0u;
        misc[kNumSurv] = 0u;
    }
    __syncthreads();

    // ---- LUT of Eq. 9 summands ------------------------------------------------------------------------
    for (int base = 0; base < nlut; base += nt * 4) {
        if (base > 0) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = base + u * nt + tid;
                ent[u] = g.table[e < nlut ? e : 0];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = base + u * nt + tid;
            if (e >= nlut) continue;
            const int m = e >> 8;
            const float b2 = sa[m * k1 + (ent[u].ij & 0xffu)];
            const float a2 = sa[m * k1 + ((ent[u].ij >> 8) & 0xffu)];
            if (MW < 0) {
                // entry = centroid pair number; its kc field holds c^2
                const int pair = e & 255;
                if (pair < (1 << g.pair_shift))
                    reinterpret_cast<float4*>(lut)[(m << g.pair_shift) + pair] = make_float4(b2, a2 - b2, ent[u].kc, 0.0f);
                continue;
            }
            // Eq. 9 rearranged: b^2 + lam (a^2 - b^2) + (lam^2 - lam) c^2, the last term folded per code value
            const float v = fmaf(ent[u].lam, a2 - b2, b2) + ent[u].kc;
            lut[e] = v;
            if (TAPS && g.lut) g.lut[(size_t)q * nlut + e] = v;
        }
    }
    __syncthreads();

    // ---- scores ---------------------------------------------------------------------------------------
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    if (nc > 0) {
        RunCursor cur;                         // positions of a thread only grow
        cur.run = 0;
        cur.next_start = run_start[1];
        cur.delta = run_src[0] - run_start[0];
        int base = 0;
        for (; base + 8 * nt <= nc; base += 8 * nt)
            score_batch<MW, 8, false, TAPS>(g, q, base, nc, tid, nt, lut, skey, run_src, run_start, cur, kmin, kmax);
        for (; base + 4 * nt <= nc; base += 4 * nt)
            score_batch<MW, 4, false, TAPS>(g, q, base, nc, tid, nt, lut, skey, run_src, run_start, cur, kmin, kmax);
        for (; base < nc; base += 4 * nt)
            score_batch<MW, 4, true, TAPS>(g, q, base, nc, tid, nt, lut, skey, run_src, run_start, cur, kmin, kmax);
    }
    if (TAPS && g.n_cand && tid == 0) g.n_cand[q] = (uint32_t)nc;
    kmin = wave_min_u32(kmin);
    kmax = wave_max_u32(kmax);
    if (lane == 0) {
        atomicMin(&misc[kMin], kmin);
        atomicMax(&misc[kMax], kmax);
    }
    __syncthreads();

    // ---- the k smallest (score, id): positions of a superset of the answer -> spos --------------------
    const int kk = k < nc ? k : nc;           // results that exist
    int nsurv;
    bool identity = false;                     // survivor e is candidate position e
    if (nc <= L.scap) {                        // few candidates: order all of them
        nsurv = nc;
        identity = true;
    } else {
        const uint32_t lo_key = misc[kMin];
        const uint32_t range = misc[kMax] - lo_key;
        const int width = 32 - __clz((int)(range | 1u));           // bits needed for range
        const int shift = width > kHistBits ? width - kHistBits : 0;   // (key - lo_key) >> shift < 1024
        const uint4* skey4 = reinterpret_cast<const uint4*>(skey);
        const int nc4 = nc >> 2;
        for (int p4 = tid; p4 < nc4; p4 += nt) {                   // four keys per LDS read
            const uint4 kq = skey4[p4];
            atomicAdd(&hist[(kq.x - lo_key) >> shift], 1u);
            atomicAdd(&hist[(kq.y - lo_key) >> shift], 1u);
            atomicAdd(&hist[(kq.z - lo_key) >> shift], 1u);
            atomicAdd(&hist[(kq.w - lo_key) >> shift], 1u);
        }
        for (int p = 4 * nc4 + tid; p < nc; p += nt) atomicAdd(&hist[(skey[p] - lo_key) >> shift], 1u);
        __syncthreads();
        // the first wavefront finds the bin bsel with count(< bsel) < kk <= count(<= bsel)
        if (tid < kWave) {
            uint32_t bsel, below, inbin;
            hist_locate(hist, (uint32_t)kk, lane, bsel, below, inbin);
            if (tid == 0) {
                misc[kSel] = bsel;
                misc[kSelCount] = below + inbin;
            }
        }
        __syncthreads();
        const uint32_t bsel = misc[kSel];
        const uint32_t count_le = misc[kSelCount];
        if (count_le <= (uint32_t)L.scap) {
            // keys of the bins <= bsel are the keys <= thr
            const unsigned long long thr64 = (unsigned long long)lo_key + (((unsigned long long)bsel + 1ull) << shift) - 1ull;
            const uint32_t thr = thr64 > 0xffffffffull ? 0xffffffffu : (uint32_t)thr64;
            for (int p4 = tid; p4 < nc4; p4 += nt) {
                const uint4 kq = skey4[p4];
                if (kq.x <= thr) spos[atomicAdd(&misc[kNumSurv], 1u)] = (uint16_t)(4 * p4);
                if (kq.y <= thr) spos[atomicAdd(&misc[kNumSurv], 1u)] = (uint16_t)(4 * p4 + 1);
                if (kq.z <= thr) spos[atomicAdd(&misc[kNumSurv], 1u)] = (uint16_t)(4 * p4 + 2);
                if (kq.w <= thr) spos[atomicAdd(&misc[kNumSurv], 1u)] = (uint16_t)(4 * p4 + 3);
            }
            for (int p = 4 * nc4 + tid; p < nc; p += nt)
                if (skey[p] <= thr) spos[atomicAdd(&misc[kNumSurv], 1u)] = (uint16_t)p;
            nsurv = (int)count_le;
        } else {
            // exact selection: k-th smallest score key, then (only if that score is tied) the ids
            uint32_t* rout = misc + kRadix;
            uint32_t* part = reinterpret_cast<uint32_t*>(lut);     // the LUT is no longer needed
            uint32_t prefix = 0, mask = 0, need = (uint32_t)kk, bucket = 0;
            const int shifts[4] = {22, 12, 2, 0};
            const int nbits[4] = {10, 10, 10, 2};
            __syncthreads();
            for (int pass = 0; pass < 4; ++pass) {
                radix_select_pass(nc, prefix, mask, shifts[pass], nbits[pass], need, hist, part, rout,
                                  [&](int p, bool& valid) { valid = true; return skey[p]; });
                prefix |= rout[0] << shifts[pass];
                mask |= ((1u << nbits[pass]) - 1u) << shifts[pass];
                need = rout[1];
                bucket = rout[2];
                __syncthreads();
            }
            const uint32_t tau = prefix;
            uint32_t id_cut = 0xffffffffu;     // among candidates with key == tau keep ids <= id_cut
            if (need < bucket) {
                uint32_t iprefix = 0, imask = 0;
                for (int pass = 0; pass < 4; ++pass) {
                    radix_select_pass(nc, iprefix, imask, shifts[pass], nbits[pass], need, hist, part, rout,
                                      [&](int p, bool& valid) {
                                          valid = skey[p] == tau;
                                          return valid ? g.ids[source_of((uint32_t)p, nr, steps, run_src, run_start)] : 0u;
                                      });
                    iprefix |= rout[0] << shifts[pass];
                    imask |= ((1u << nbits[pass]) - 1u) << shifts[pass];
                    need = rout[1];
                    __syncthreads();
                }
                id_cut = iprefix;
            }
            for (int p = tid; p < nc; p += nt) {
                const uint32_t key = skey[p];
                if (key > tau) continue;
                if (key == tau && id_cut != 0xffffffffu &&
                    g.ids[source_of((uint32_t)p, nr, steps, run_src, run_start)] > id_cut)
                    continue;
                spos[atomicAdd(&misc[kNumSurv], 1u)] = (uint16_t)p;
            }
            nsurv = kk;
        }
    }
    __syncthreads();

    // ---- fetch the survivors' ids: 64-bit keys (score bits, id) --------------------------------------------
    for (int e = tid; e < nsurv; e += nt) {
        const uint32_t p = identity ? (uint32_t)e : (uint32_t)spos[e];
        const uint32_t id = g.ids[source_of(p, nr, steps, run_src, run_start)];
        surv[e] = ((unsigned long long)skey[p] << 32) | id;
    }
    __syncthreads();

    // ---- order the survivors, write the first k ---------------------------------------------------------
    if (nsurv <= kCountRankMax) {
        // rank = number of smaller keys (keys are unique); four adjacent lanes share one survivor
        const int sub = tid & 3;
        for (int e0 = 0; e0 < nsurv; e0 += nt / 4) {
            const int e = e0 + (tid >> 2);
            const bool valid = e < nsurv;
            const unsigned long long key = valid ? surv[e] : 0ull;
            uint32_t rank = 0;
            for (int j = sub; j < nsurv; j += 4) rank += (surv[j] < key) ? 1u : 0u;
            rank += quad_swap1(rank);
            rank += quad_swap2(rank);
            if (valid && sub == 0 && rank < (uint32_t)k) {
                g.out_ids[(size_t)q * k + rank] = (int64_t)(uint32_t)key;
                g.out_dists[(size_t)q * k + rank] = mono_inv((uint32_t)(key >> 32));
            }
        }
    } else {
        const int npad = next_pow2(nsurv);
        for (int e = nsurv + tid; e < npad; e += nt) surv[e] = ~0ull;
        bitonic_sort_lds(surv, npad, tid, nt);
        for (int e = tid; e < kk; e += nt) {
            const unsigned long long key = surv[e];
            g.out_ids[(size_t)q * k + e] = (int64_t)(uint32_t)key;
            g.out_dists[(size_t)q * k + e] = mono_inv((uint32_t)(key >> 32));
        }
    }
    for (int e = kk + tid; e < k; e += nt) {
        g.out_ids[(size_t)q * k + e] = (int64_t)-1;
        g.out_dists[(size_t)q * k + e] = __builtin_inff();
    }
}

template <bool TAPS, bool FUSED>
static void launch_rerank_t(const RerankArgs& a, const RerankLds& L, const RankArgs& rk, const RankOffsets& RL,
                            hipStream_t s) {
    const dim3 grid((unsigned)(a.nq + a.early)), block(a.threads);
    if (a.code_format == 1) {
        // word-wise variants for the plain entry point; the tapped one takes the byte-wise kernel
        switch (TAPS || a.M % 2 ? 0 : a.M / 2) {
            case 2: hipLaunchKernelGGL((rerank_kernel<TAPS ? kPairLambda : -2, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
            case 4: hipLaunchKernelGGL((rerank_kernel<TAPS ? kPairLambda : -4, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
            case 8: hipLaunchKernelGGL((rerank_kernel<TAPS ? kPairLambda : -8, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
            default: hipLaunchKernelGGL((rerank_kernel<kPairLambda, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
        }
        return;
    }
    switch ((a.M % 4 == 0) ? a.M / 4 : 0) {
        case 1: hipLaunchKernelGGL((rerank_kernel<1, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
        case 2: hipLaunchKernelGGL((rerank_kernel<2, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
        case 4: hipLaunchKernelGGL((rerank_kernel<4, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
        case 8: hipLaunchKernelGGL((rerank_kernel<8, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
        default: hipLaunchKernelGGL((rerank_kernel<0, TAPS, FUSED>), grid, block, L.total, s, a, L, rk, RL); break;
    }
}

int rerank_fused_tuples_per_thread() { return kFusedPer; }

hipError_t launch_rerank(const RerankArgs& a_in, const RankArgs* fused, hipStream_t s) {
    if (a_in.nq <= 0) return hipSuccess;
    RerankArgs a = a_in;
    a.pair_shift = pair_table_shift(a.k1);
    const bool taps = a.n_cand || a.cand_ids || a.scores || a.lut;
    RankArgs rk = {};
    RankOffsets RL = {};
    if (fused) {
        if (taps || fused->P != 2) return hipErrorInvalidValue;
        rk = *fused;
        RL = rank_offsets(rk.P, rk.R, rk.T, rk.hashed);
        if (RL.Tcap > rerank_fused_tuples_per_thread() * a.threads) return hipErrorInvalidValue;
    }
    if (a.code_format == 1 && a.lut) return hipErrorInvalidValue;      // that tap is the one-byte format's table
    const RerankLds L = rerank_layout(a.M, a.k1, a.T, a.C, a.k, a.threads, fused ? RL.total : 0, a.code_format);
    if (fused) launch_rerank_t<false, true>(a, L, rk, RL, s);
    else if (taps) launch_rerank_t<true, false>(a, L, rk, RL, s);
    else launch_rerank_t<false, false>(a, L, rk, RL, s);
    return hipGetLastError();
}

hipError_t configure_rerank(size_t max_dynamic_lds) {
    const void* kernels[] = {
        reinterpret_cast<const void*>(rerank_kernel<0, false, false>), reinterpret_cast<const void*>(rerank_kernel<1, false, false>),
        reinterpret_cast<const void*>(rerank_kernel<2, false, false>), reinterpret_cast<const void*>(rerank_kernel<4, false, false>),
        reinterpret_cast<const void*>(rerank_kernel<8, false, false>), reinterpret_cast<const void*>(rerank_kernel<0, true, false>),
        reinterpret_cast<const void*>(rerank_kernel<1, true, false>),  reinterpret_cast<const void*>(rerank_kernel<2, true, false>),
        reinterpret_cast<const void*>(rerank_kernel<4, true, false>),  reinterpret_cast<const void*>(rerank_kernel<8, true, false>),
        reinterpret_cast<const void*>(rerank_kernel<0, false, true>),  reinterpret_cast<const void*>(rerank_kernel<1, false, true>),
        reinterpret_cast<const void*>(rerank_kernel<2, false, true>),  reinterpret_cast<const void*>(rerank_kernel<4, false, true>),
        reinterpret_cast<const void*>(rerank_kernel<8, false, true>),
        reinterpret_cast<const void*>(rerank_kernel<kPairLambda, false, false>),
        reinterpret_cast<const void*>(rerank_kernel<kPairLambda, true, false>),
        reinterpret_cast<const void*>(rerank_kernel<kPairLambda, false, true>),
        reinterpret_cast<const void*>(rerank_kernel<-2, false, false>), reinterpret_cast<const void*>(rerank_kernel<-2, false, true>),
        reinterpret_cast<const void*>(rerank_kernel<-4, false, false>), reinterpret_cast<const void*>(rerank_kernel<-4, false, true>),
        reinterpret_cast<const void*>(rerank_kernel<-8, false, false>), reinterpret_cast<const void*>(rerank_kernel<-8, false, true>)};
    for (const void* kfn : kernels) {
        hipFuncAttributes attr;
        hipError_t e = hipFuncGetAttributes(&attr, kfn);
        if (e != hipSuccess) return e;
        if (attr.sharedSizeBytes != 0) return hipErrorInvalidValue;   // the LUT must start at LDS address 0
        e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace pqt
