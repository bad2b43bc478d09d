// Device code of the re-rank kernel: vector proposal, re-ranking by line quantisation and the final ordering
// (Sec. 3.2 "vector proposal", Sec. 3.3 "Online computation" Eq. 8-9, Sec. 4 last kernel).
//
// One workgroup per query.
//   * the per-query table LUT[m][c] of Eq. 9 summands is built in LDS from the level-1
//     sub-part distances the traversal already produced (no new distance is computed);
//   * codes are stored bin-major beside the ids, so the candidates of a proposed slot are one
//     contiguous run.  A wavefront scores a contiguous piece of the candidate list, 64 positions
//     (one window) after the other, consecutive lanes reading consecutive codes (coalesced),
//     eight windows in flight; where runs are long (eight candidates or more on average) it
//     walks the run list as one, with scalar control and one compare and select per run boundary,
//     where they are short every thread searches the list for its own position.  The id array is
//     only touched for the few survivors;
//   * score = sum over m = 0..M-1, in that order, of LUT[m][code[m]] in fp32;
//   * a thread scores at most twenty candidates and keeps their keys (ordered score bits) in
//     registers through the selection: with eight workgroups per compute unit the vector ALU is
//     busy most of the time on a cache-resident index, so what counts is the number of vector
//     instructions per candidate and how many queries a compute unit has in flight, which is set
//     by the LDS a workgroup holds -- a key array in LDS would double it;
//   * the k best by (score, id): one 1024-bin histogram over the ordered score bits between the
//     smallest and largest score of the query; the first wavefront locates the bin b that holds the
//     k-th smallest; the keys in bins <= b (a superset of the answer, normally a few more
//     than k) are appended to a short list with their positions, their ids fetched, and the
//     (score bits, id) keys sorted in registers.  If the superset does not fit (heavily tied
//     scores) an exact radix select on score bits, then on ids, picks exactly k.
#pragma once
#include <type_traits>

#include "rank_head_device.hpp"
#include "rerank_variants.hpp"

namespace pqt {


constexpr int kCountRankMax = 32;    // survivors ordered by counting ranks up to this many, else sorted
constexpr int kWalkMinRun = 8;       // mean run length from which a wavefront walks the run list together
constexpr int kRunPrefetch = 64;     // runs fetched before the run count is known

// The run list of one query: the first rcap runs in LDS, any further ones in memory.  The LDS arrays
// are named by their byte addresses (the kernels here have no static LDS, so the dynamic LDS starts
// at address 0; the launcher checks that).
typedef __attribute__((address_space(3))) const uint32_t lds_cuint;
struct RunList {
    uint32_t src, start;       // LDS addresses of run_src / run_start
    const uint2* mem;          // runs of this query in memory
    int rcap, nr;
    uint32_t nc;
    __device__ __forceinline__ uint32_t start_at(int r) const {   // r <= nr
        return r < rcap || r == nr && nr <= rcap ? *reinterpret_cast<lds_cuint*>((uintptr_t)(start + 4u * (uint32_t)r))
                                                 : (r < nr ? mem[r].y : nc);
    }
    __device__ __forceinline__ uint32_t src_at(int r) const {     // r < nr
        return r < rcap ? *reinterpret_cast<lds_cuint*>((uintptr_t)(src + 4u * (uint32_t)r)) : mem[r].x;
    }
};

// Position p of the candidate list -> position in ids/codes: the run r with
// start(r) <= p < start(r+1), found in `steps` = ceil(log2(nr)) halvings.
__device__ __forceinline__ uint32_t source_of(uint32_t p, int steps, const RunList& R) {
    int lo = 0, hi = R.nr;
    for (int s = 0; s < steps; ++s) {
        const int mid = (lo + hi) >> 1;
        const bool ge = R.start_at(mid) <= p;
        lo = ge ? mid : lo;
        hi = ge ? hi : mid;
    }
    return R.src_at(lo) + (p - R.start_at(lo));
}

// One pass of a most-significant-digit radix select (exact fallback).  Counts, among the items whose
// key agrees with `prefix` on the bits of `mask`, the digit (key >> shift) & (2^bits - 1); finds the
// digit holding the item of 1-based rank `need`.  out[0] = digit, out[1] = rank inside it, out[2] =
// size of the chosen digit's bucket.  each_key(f) calls f(key) for every item of the calling thread.
// All threads must call it; ends with a barrier.
template <typename EachKey>
__device__ __forceinline__ void radix_select_pass(uint32_t prefix, uint32_t mask, int shift, int bits, uint32_t need,
                                                  uint32_t* hist, uint32_t* part, uint32_t* out, EachKey each_key) {
    const int tid = threadIdx.x, nt = blockDim.x;
    const int nb = 1 << bits;
    for (int e = tid; e < nb; e += nt) hist[e] = 0;
    __syncthreads();
    each_key([&](uint32_t key) {
        if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
    });
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
// the same for byte B of a code word: four times the byte in ONE sub-dword shift, for the low byte too
// (for which the compiler would shift the whole word and mask)
template <int B>
__device__ __forceinline__ float lut_at_byte(int m, uint32_t word) {
    uint32_t addr;
    if constexpr (B == 0)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0"
            : "=v"(addr) : "v"(2u), "v"(word));
    else
        addr = ((word >> (8 * B)) & 0xffu) << 2;
    return *reinterpret_cast<lds_cfloat*>((uintptr_t)(addr + (uint32_t)m * 1024u));
}

// The run a thread's current candidate position lies in, kept in registers: positions of a thread
// only grow, so the run only moves forwards and the run list is read only when a position crosses
// into another run.
struct RunCursor {
    int run;
    uint32_t next_start;   // run_start[run + 1]
    uint32_t delta;        // run_src[run] - run_start[run]: position in ids/codes = candidate position + delta
};

// Where a wavefront stands in the run list while it walks its piece of the candidate list, 64
// positions (one window) at a time.  Lane l holds run blk0 + l of the list; r (the same in every
// lane) is the first run that starts after the windows done so far, dcur the offset
// run_src - run_start of run r - 1.  Everything that steers the walk is wavefront-uniform, so the
// per-position work is one compare and one select per run boundary inside the window.
struct WaveRuns {
    uint32_t v_src, v_start;   // run blk0 + lane (v_start = 0xffffffff past the end of the list)
    int blk0, r;
    uint32_t dcur;
    uint32_t next_s;           // start of run r, 0xffffffff when the list is used up
    __device__ __forceinline__ void load(const RunList& R, int first, int lane) {
        blk0 = first;
        const int idx = first + lane;
        v_start = 0xffffffffu;
        v_src = 0u;
        if (idx < R.nr) {
            v_start = R.start_at(idx);
            v_src = R.src_at(idx);
        }
    }
    __device__ __forceinline__ void fetch_next(const RunList& R, int lane) {
        if (r >= R.nr) {
            next_s = 0xffffffffu;
            return;
        }
        if (r - blk0 >= kWave) load(R, r & ~(kWave - 1), lane);
        next_s = (uint32_t)__builtin_amdgcn_readlane((int)v_start, r - blk0);
    }
    // positions [wbase, ...) come next: r = number of runs that start at or before wbase (at least one)
    __device__ __forceinline__ void seek(const RunList& R, uint32_t wbase, int lane) {
        int b = 0;
        while ((b + 1) * kWave < R.nr &&
               (uint32_t)__builtin_amdgcn_readfirstlane((int)R.start_at((b + 1) * kWave)) <= wbase)
            ++b;
        load(R, b * kWave, lane);
        const int cnt = __popcll(__ballot(v_start <= wbase));
        r = b * kWave + cnt;
        dcur = (uint32_t)__builtin_amdgcn_readlane((int)(v_src - v_start), cnt > 0 ? cnt - 1 : 0);
        fetch_next(R, lane);
    }
    // offset of every lane's position wb + lane (wb: multiple of 64, not below the last window's);
    // a window without a run boundary costs one scalar compare
    __device__ __forceinline__ uint32_t window(const RunList& R, uint32_t wb, int lane) {
        uint32_t delta = dcur;
        while (next_s < wb + kWave) {
            const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)v_src, r - blk0) - next_s;
            delta = wb + (uint32_t)lane >= next_s ? d : delta;
            dcur = d;
            ++r;
            fetch_next(R, lane);
        }
        return delta;
    }
};

// (pair, lambda level) codes: the summand of Eq. 9 for one sub-part from the pair's LDS entry
// (b^2, a^2 - b^2, c^2) and the level; lambda = (level - 96) / 16 is exact in fp32.
constexpr int kPairLambda = -1;      // MW < 0 selects this code format: -1 any M (byte loads), else -(words per code)
__device__ __forceinline__ float pair_lambda_term(const float4* plut, int shift, int m, uint32_t pair, uint32_t level) {
    const float4 e = plut[(m << shift) + pair];
    const float lam = fmaf((float)level, 0.0625f, -6.0f);
    return fmaf(fmaf(lam, lam, -lam), e.z, fmaf(lam, e.y, e.x));
}

// Scores U candidate positions per thread (wb + u * 64 + lane: a wavefront walks its own contiguous
// piece of the candidate list, U windows of 64 positions at a time) and leaves their keys (ordered
// score bits) in key[0..U).  CHECK: positions may reach pend (their keys are left alone).
// WALK: the wavefront walks the run list (long runs); else every thread searches it (short runs).
template <int MW, int U, bool CHECK, bool TAPS, bool WALK>
__device__ __forceinline__ void score_batch(const RerankArgs& g, int64_t q, int wb, int lane, int pend,
                                            const float* lut, uint32_t* key, const RunList& R, WaveRuns& wr,
                                            RunCursor& cur, uint32_t& kmin, uint32_t& kmax) {
    const int p0 = wb + lane;
    constexpr int NW = MW > 0 ? MW : (MW < -1 ? -MW : 0);      // code words fetched up front (0: byte loads)
    const int M = MW > 0 ? 4 * MW : (MW < -1 ? -2 * MW : g.M);
    uint32_t src[U];
    uint32_t cw[U][NW > 0 ? NW : 1];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t p = (uint32_t)(p0 + u * kWave);
        if (WALK) {
            const uint32_t delta = wr.window(R, (uint32_t)(wb + u * kWave), lane);
            // a position past the end reads the first candidate of a run the wavefront holds
            src[u] = (!CHECK || p < (uint32_t)pend) ? p + delta : (uint32_t)__builtin_amdgcn_readlane((int)wr.v_src, 0);
        } else if (!CHECK || p < (uint32_t)pend) {
            if (p >= cur.next_start) {
                // usually the next run; otherwise the run is found by halving what is left of the list
                // (a thread's first position, or short runs: a step of 64 positions passes several)
                int lo = cur.run + 1;
                uint32_t next = R.start_at(lo + 1);
                if (p >= next) {
                    int hi = R.nr;                                  // start_at(lo) <= p < start_at(hi) = nc
                    ++lo;
                    while (hi - lo > 1) {
                        const int mid = (lo + hi) >> 1;
                        const bool ge = R.start_at(mid) <= p;
                        lo = ge ? mid : lo;
                        hi = ge ? hi : mid;
                    }
                    next = R.start_at(lo + 1);
                }
                cur.run = lo;
                cur.next_start = next;
                cur.delta = R.src_at(lo) - R.start_at(lo);
            }
            src[u] = p + cur.delta;
        } else {
            src[u] = R.src_at(0);
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
        const int p = p0 + u * kWave;
        if (CHECK && p >= pend) continue;
        float s;
        if (MW > 0) {
            s = lut_at_byte<0>(0, cw[u][0]);               // sum in ascending m
            s += lut_at_byte<1>(1, cw[u][0]);
            s += lut_at_byte<2>(2, cw[u][0]);
            s += lut_at_byte<3>(3, cw[u][0]);
#pragma unroll
            for (int j = 1; j < MW; ++j) {
                const uint32_t wv = cw[u][j];
                s += lut_at_byte<0>(j * 4 + 0, wv);
                s += lut_at_byte<1>(j * 4 + 1, wv);
                s += lut_at_byte<2>(j * 4 + 2, wv);
                s += lut_at_byte<3>(j * 4 + 3, wv);
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
        const uint32_t ky = mono_key(s);
        key[u] = ky;
        kmin = min(kmin, ky);
        kmax = max(kmax, ky);
        if (TAPS) {
            if (g.scores) g.scores[(size_t)q * g.C + p] = s;
            if (g.cand_ids) g.cand_ids[(size_t)q * g.C + p] = (int64_t)g.ids[src[u]];
        }
    }
}

// MW = 32-bit words per code (M/4) for M in {4, 8, 16, 32}; 0 = any other M (byte loads);
// MW < 0 = codes hold (centroid pair, lambda level) per sub-part, scored by Eq. 9 directly.
// FUSED: a query whose meta.x is kMetaTodo (the ranking head pass could not finish it) is first
// ranked in full by this workgroup.
template <int MW, bool TAPS, bool FUSED>
__global__ __launch_bounds__(1024, TAPS ? 1 : ((MW >= 8 || MW <= -8) ? 4 : 8)) void rerank_kernel(RerankArgs g, RerankLds L, RankArgs rk, RankOffsets RL) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* surv = reinterpret_cast<unsigned long long*>(smem + L.surv);
    float* lut = reinterpret_cast<float*>(smem);                 // L.lut == 0
    float* sa = reinterpret_cast<float*>(smem + L.a);
    uint32_t* run_src = reinterpret_cast<uint32_t*>(smem + L.run_src);
    uint32_t* run_start = reinterpret_cast<uint32_t*>(smem + L.run_start);
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
    uint32_t* part = reinterpret_cast<uint32_t*>(smem + L.part);
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
    if (FUSED && meta.x == kMetaTodo) {        // same for the whole workgroup
        // the run list goes to memory (this query's own rows), the counts come back through LDS.
        // First the head pass's third level (128 tuples) by the first wavefront alone: few vector
        // instructions, and nearly every left-over query is finished by it; the full ranking by the
        // whole workgroup only if even those runs do not fill the candidate budget.
        bool ranked = false;
        if (g.mid_T1 > 0) {
            if (tid < kWave) {
                HeadLds& S = *reinterpret_cast<HeadLds*>(smem);
                const int R1 = rk.R < kHeadT ? rk.R : kHeadT;
                head_load_lists(rk, S, q, lane, R1);
                unsigned long long carry = ~0ull;
                const int r = head_level<2, true>(rk, S, q, lane, R1, g.mid_T1, 0, g.mid_npairs, RL.Tcap, true, carry, misc + kRanked);
                if (lane == 0) misc[kRanked + 2] = r == 1 ? 1u : 0u;
            }
            __syncthreads();
            ranked = misc[kRanked + 2] != 0u;
            __syncthreads();
        }
        if (!ranked) rank_query<2, true, kFusedPer, 0>(rk, RL, q, smem, misc + kRanked);
        meta = make_uint2(misc[kRanked], misc[kRanked + 1]);
    }
    const uint2* qruns = g.runs + (size_t)q * T;

    // ---- issue every load that needs no other result first ------------------------------------------
    uint2 run0 = make_uint2(0u, 0u);
    if (tid < kRunPrefetch && tid < L.rcap) run0 = qruns[tid];
    // table entries: a thread takes code value c = tid mod 256 of the sub-parts m0, m0 + ms, ... (m0 and ms
    // are the same for a wavefront, so which sub-parts exist is decided by scalar code)
    const int lut_c = tid & 255;
    const int lut_m0 = __builtin_amdgcn_readfirstlane(tid >> 8), lut_ms = nt >> 8;
    const int Mlut = MW > 0 ? 4 * MW : (MW < -1 ? -2 * MW : M);
    // entries a thread fetches per round: with codes of up to eight bytes all of a thread's entries at once, so
    // that no load is waited for inside the table phase (256 threads had two rounds of four)
    constexpr int kEnt = (MW > 0 && MW <= 2) ? 8 : 4;
    constexpr bool kOneRound = MW > 0 && 4 * MW <= kEnt;
    CodeEntry ent[kEnt];
#pragma unroll
    for (int u = 0; u < kEnt; ++u) {
        const int m = lut_m0 + u * lut_ms;
        ent[u] = g.table[(m < Mlut ? m : 0) * 256 + lut_c];
    }
    for (int e = tid; e < M * k1; e += nt) sa[e] = g.a[(size_t)q * M * k1 + e];
    for (int e = tid; e < kHistSize; e += nt) hist[e] = 0;
    const int nr = __builtin_amdgcn_readfirstlane((int)meta.x);     // the same in every thread
    const int nc = __builtin_amdgcn_readfirstlane((int)meta.y);
    int steps = 0;
    while ((1 << steps) < nr) ++steps;
    const int nr_lds = nr < L.rcap ? nr : L.rcap;
    if (tid < kRunPrefetch && tid < nr_lds) {
        run_src[tid] = run0.x;
        run_start[tid] = run0.y;
    }
    for (int r = kRunPrefetch + tid; r < nr_lds; r += nt) {
        const uint2 run = qruns[r];
        run_src[r] = run.x;
        run_start[r] = run.y;
    }
    if (tid == 0) {
        if (nr <= L.rcap) run_start[nr] = (uint32_t)nc;
        misc[kMin] = 0xffffffffu;
        misc[kMax] = 0u;
        misc[kNumSurv] = 0u;
    }
    RunList R;
    R.src = L.run_src; R.start = L.run_start; R.mem = qruns; R.rcap = L.rcap; R.nr = nr; R.nc = (uint32_t)nc;
    __syncthreads();

    // ---- LUT of Eq. 9 summands ------------------------------------------------------------------------
    auto table_entry = [&](int m, const CodeEntry& ce) {
        const int e = m * 256 + lut_c;
        const float* sam = sa + m * k1;
        const float b2 = sam[ce.ij & 0xffu];
        const float a2 = sam[(ce.ij >> 8) & 0xffu];
        if (MW < 0) {
            // entry = centroid pair number; its kc field holds c^2
            if (lut_c < (1 << g.pair_shift))
                reinterpret_cast<float4*>(lut)[(m << g.pair_shift) + lut_c] = make_float4(b2, a2 - b2, ce.kc, 0.0f);
            return;
        }
        // Eq. 9 rearranged: b^2 + lam (a^2 - b^2) + (lam^2 - lam) c^2, the last term folded per code value
        const float v = fmaf(ce.lam, a2 - b2, b2) + ce.kc;
        lut[e] = v;
        if (TAPS && g.lut) g.lut[(size_t)q * nlut + e] = v;
    };
    if constexpr (kOneRound) {
#pragma unroll
        for (int u = 0; u < kEnt; ++u) {
            const int m = lut_m0 + u * lut_ms;
            if (m < Mlut) table_entry(m, ent[u]);
        }
    } else {
        for (int mb = lut_m0; mb < Mlut; mb += 4 * lut_ms) {
            CodeEntry cur_ent[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) cur_ent[u] = ent[u];
            if (mb + 4 * lut_ms < Mlut) {          // the next round's entries are fetched while this one is worked on
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int m = mb + (4 + u) * lut_ms;
                    ent[u] = g.table[(m < Mlut ? m : 0) * 256 + lut_c];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int m = mb + u * lut_ms;
                if (m < Mlut) table_entry(m, cur_ent[u]);      // (no early exit: the loop must unroll in full)
            }
        }
    }
    __syncthreads();

    // ---- scores: wavefront v owns positions [v * chunk, (v + 1) * chunk); position pos0 + u * 64 -> key[u] -----
    const int chunk = ((nc + (nt >> 6) - 1) / (nt >> 6) + kWave - 1) & ~(kWave - 1);     // <= 64 * kKeysPerThread
    const int pos0 = (tid >> 6) * chunk + lane;
    const int pend = min(nc, ((tid >> 6) + 1) * chunk);      // this wavefront's positions end here
    uint32_t key[kKeysPerThread];
#pragma unroll
    for (int u = 0; u < kKeysPerThread; ++u) key[u] = 0xffffffffu;
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    if (nc > 0) {
        const int wbase = __builtin_amdgcn_readfirstlane(pos0 - lane);    // the same for a wavefront
        // eight positions in flight per thread; four when a code has four or more words or holds (pair, lambda)
        // tuples, whose scoring needs the registers
        constexpr int UB = (MW >= 4 || MW <= -2) ? 4 : 8;
        static_assert(kKeysPerThread % 4 == 0, "batches of four or eight");
        WaveRuns wr;
        RunCursor cur;                         // positions of a thread only grow
        auto score_all = [&](auto walk) {
            constexpr bool WALK = decltype(walk)::value;
#pragma unroll
            for (int b = 0; b * UB + UB <= kKeysPerThread; ++b) {
                const int base = wbase + b * UB * kWave;
                if (base + UB * kWave <= pend)
                    score_batch<MW, UB, false, TAPS, WALK>(g, q, base, lane, pend, lut, key + b * UB, R, wr, cur, kmin, kmax);
                else if (base < pend)
                    score_batch<MW, UB, true, TAPS, WALK>(g, q, base, lane, pend, lut, key + b * UB, R, wr, cur, kmin, kmax);
            }
            if (kKeysPerThread % UB) {         // a last batch of four
                constexpr int done = kKeysPerThread / UB * UB;
                const int base = wbase + done * kWave;
                if (base + 4 * kWave <= pend)
                    score_batch<MW, 4, false, TAPS, WALK>(g, q, base, lane, pend, lut, key + done, R, wr, cur, kmin, kmax);
                else if (base < pend)
                    score_batch<MW, 4, true, TAPS, WALK>(g, q, base, lane, pend, lut, key + done, R, wr, cur, kmin, kmax);
            }
        };
        if (nr * kWalkMinRun <= nc) {          // runs long enough that a window of 64 positions meets few of them
            wr.seek(R, (uint32_t)wbase, lane);
            score_all(std::true_type{});
        } else {
            cur.run = 0;
            cur.next_start = R.start_at(1);
            cur.delta = R.src_at(0) - R.start_at(0);
            score_all(std::false_type{});
        }
    }
    if (TAPS && g.n_cand && tid == 0) g.n_cand[q] = (uint32_t)nc;
    kmin = wave_min_u32(kmin);
    kmax = wave_max_u32(kmax);
    if (lane == 0) {
        atomicMin(&misc[kMin], kmin);
        atomicMax(&misc[kMax], kmax);
    }
    __syncthreads();

    // ---- the k smallest (score, id): (key, position) of a superset of the answer -> surv ---------------
    const int kk = k < nc ? k : nc;           // results that exist
    int nsurv;
    bool by_bin = false;                       // the survivors can be placed by their histogram bin (see below)
    uint32_t lo_key = 0;
    int shift = 0;
    if (nc <= L.scap) {                        // few candidates: order all of them
#pragma unroll
        for (int u = 0; u < kKeysPerThread; ++u) {
            const int p = pos0 + u * kWave;
            if (p < pend) surv[p] = ((unsigned long long)key[u] << 32) | (uint32_t)p;
        }
        nsurv = nc;
    } else {
        lo_key = misc[kMin];
        const uint32_t range = misc[kMax] - lo_key;
        const int width = 32 - __clz((int)(range | 1u));           // bits needed for range
        shift = width > kHistBits ? width - kHistBits : 0;          // (key - lo_key) >> shift < 1024
#pragma unroll
        for (int u = 0; u < kKeysPerThread; ++u) {
            if (u * kWave >= chunk) break;                             // same for the whole workgroup
            if (pos0 + u * kWave < pend) atomicAdd(&hist[(key[u] - lo_key) >> shift], 1u);
        }
        __syncthreads();
        // counts -> first positions, in place (a prefix sum by the whole workgroup); the thread that owns the
        // bin bsel with count(< bsel) < kk <= count(<= bsel) notes it
        {
            const int bpt = kHistSize / nt;                        // 4, 2 or 1 bins per thread
            uint32_t sum = 0;
            for (int j = 0; j < bpt; ++j) sum += hist[tid * bpt + j];
            uint32_t total;
            uint32_t c = block_exclusive_sum(sum, part, total);
            for (int j = 0; j < bpt; ++j) {
                const uint32_t cnt = hist[tid * bpt + j];
                hist[tid * bpt + j] = c;
                if (c < (uint32_t)kk && (uint32_t)kk <= c + cnt) {
                    misc[kSel] = (uint32_t)(tid * bpt + j);
                    misc[kSelCount] = c + cnt;
                }
                c += cnt;
            }
        }
        __syncthreads();
        const uint32_t bsel = misc[kSel];
        const uint32_t count_le = misc[kSelCount];
        if (count_le <= (uint32_t)L.scap) {
            // keys of the bins <= bsel are the keys <= thr
            const unsigned long long thr64 = (unsigned long long)lo_key + (((unsigned long long)bsel + 1ull) << shift) - 1ull;
            const uint32_t thr = thr64 > 0xffffffffull ? 0xffffffffu : (uint32_t)thr64;
            by_bin = thr != 0xffffffffu && count_le <= (uint32_t)nt;
            if (thr != 0xffffffffu) {
                // key slots without a candidate hold 0xffffffff > thr.  A wavefront counts its keys <= thr,
                // reserves room for them with one atomic, then writes them: no wait for LDS per window
                uint32_t mine = 0;
#pragma unroll
                for (int u = 0; u < kKeysPerThread; ++u) mine += (uint32_t)__popcll(__ballot(key[u] <= thr));
                uint32_t at = 0;
                if (lane == 0 && mine) at = atomicAdd(&misc[kNumSurv], mine);
                at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
#pragma unroll
                for (int u = 0; u < kKeysPerThread; ++u) {
                    const unsigned long long hm = __ballot(key[u] <= thr);
                    if (hm == 0ull) continue;                          // the same for the wavefront
                    if (key[u] <= thr) {
                        const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(hm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)hm, 0u));
                        surv[at + below] = ((unsigned long long)key[u] << 32) | (uint32_t)(pos0 + u * kWave);
                    }
                    at += (uint32_t)__popcll(hm);
                }
            } else {
#pragma unroll
                for (int u = 0; u < kKeysPerThread; ++u) {
                    const int p = pos0 + u * kWave;
                    if (u * kWave >= chunk) break;
                    if (p < pend && key[u] <= thr)
                        surv[atomicAdd(&misc[kNumSurv], 1u)] = ((unsigned long long)key[u] << 32) | (uint32_t)p;
                }
            }
            nsurv = (int)count_le;
        } else {
            // exact selection: k-th smallest score key, then (only if that score is tied) the ids
            uint32_t* rout = misc + kRadix;
            uint32_t prefix = 0, mask = 0, need = (uint32_t)kk, bucket = 0;
            const int shifts[4] = {22, 12, 2, 0};
            const int nbits[4] = {10, 10, 10, 2};
            __syncthreads();
            for (int pass = 0; pass < 4; ++pass) {
                radix_select_pass(prefix, mask, shifts[pass], nbits[pass], need, hist, part, rout, [&](auto f) {
#pragma unroll
                    for (int u = 0; u < kKeysPerThread; ++u)
                        if (pos0 + u * kWave < pend) f(key[u]);
                });
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
                    radix_select_pass(iprefix, imask, shifts[pass], nbits[pass], need, hist, part, rout, [&](auto f) {
#pragma unroll
                        for (int u = 0; u < kKeysPerThread; ++u) {
                            const int p = pos0 + u * kWave;
                            if (p < pend && key[u] == tau) f(g.ids[source_of((uint32_t)p, steps, R)]);
                        }
                    });
                    iprefix |= rout[0] << shifts[pass];
                    imask |= ((1u << nbits[pass]) - 1u) << shifts[pass];
                    need = rout[1];
                    __syncthreads();
                }
                id_cut = iprefix;
            }
#pragma unroll
            for (int u = 0; u < kKeysPerThread; ++u) {
                const int p = pos0 + u * kWave;
                if (p >= pend || key[u] > tau) continue;
                if (key[u] == tau && id_cut != 0xffffffffu && g.ids[source_of((uint32_t)p, steps, R)] > id_cut) continue;
                surv[atomicAdd(&misc[kNumSurv], 1u)] = ((unsigned long long)key[u] << 32) | (uint32_t)p;
            }
            nsurv = kk;
        }
    }
    __syncthreads();

    // ---- usual case: the survivors are placed by their histogram bin, no sort -----------------------------
    // hist[] holds the first position of every bin among the sorted keys.  A thread takes one survivor,
    // fetches its id, and drops the (score bits, id) key into its bin's range with one LDS atomic; then every
    // key counts the smaller keys of its own bin (one to four entries) and that is its place in the output.
    if (by_bin) {
        const bool have = tid < nsurv;
        unsigned long long mine = ~0ull;
        uint32_t bin = 0;
        if (have) {
            const unsigned long long kp = surv[tid];
            mine = (kp & 0xffffffff00000000ull) | g.ids[source_of((uint32_t)kp, steps, R)];
            bin = ((uint32_t)(kp >> 32) - lo_key) >> shift;
        }
        __syncthreads();                       // every surv[] entry has been read
        if (have) surv[atomicAdd(&hist[bin], 1u)] = mine;
        __syncthreads();                       // hist[b] is now the end of bin b, the start of bin b + 1
        if (have) {
            const uint32_t first = bin ? hist[bin - 1] : 0u, end = hist[bin];
            uint32_t r = first;
            for (uint32_t x = first; x < end; ++x) r += surv[x] < mine ? 1u : 0u;
            if (r < (uint32_t)kk) {
                g.out_ids[(size_t)q * k + r] = (int64_t)(uint32_t)mine;
                g.out_dists[(size_t)q * k + r] = mono_inv((uint32_t)(mine >> 32));
            }
        }
        for (int e = kk + tid; e < k; e += nt) {
            g.out_ids[(size_t)q * k + e] = (int64_t)-1;
            g.out_dists[(size_t)q * k + e] = __builtin_inff();
        }
        return;
    }

    // ---- otherwise: fetch the survivors' ids: 64-bit keys (score bits, id) ------------------------------
    // (one round of loads for the whole list: the thread that holds a surviving key does not fetch the id
    // itself, or a wavefront would wait for memory once per key slot)
    for (int e = tid; e < nsurv; e += nt) {
        const unsigned long long kp = surv[e];
        const uint32_t id = g.ids[source_of((uint32_t)kp, steps, R)];
        surv[e] = (kp & 0xffffffff00000000ull) | id;
    }
    __syncthreads();

    // ---- order the survivors, write the first k ---------------------------------------------------------
    if (nsurv <= kCountRankMax) {
        // a handful: rank = number of smaller keys (keys are unique); four adjacent lanes share one survivor
        const int sub = tid & 3;
        for (int e0 = 0; e0 < nsurv; e0 += nt / 4) {
            const int e = e0 + (tid >> 2);
            const bool valid = e < nsurv;
            const unsigned long long skey = valid ? surv[e] : 0ull;
            uint32_t rank = 0;
            for (int j = sub; j < nsurv; j += 4) rank += (surv[j] < skey) ? 1u : 0u;
            rank += quad_swap1(rank);
            rank += quad_swap2(rank);
            if (valid && sub == 0 && rank < (uint32_t)k) {
                g.out_ids[(size_t)q * k + rank] = (int64_t)(uint32_t)skey;
                g.out_dists[(size_t)q * k + rank] = mono_inv((uint32_t)(skey >> 32));
            }
        }
    } else {
        // sorted in registers, 64 keys per wavefront (comparisons grow as n log^2 n, not n^2)
        const int npad = next_pow2(nsurv) < kWave ? kWave : next_pow2(nsurv);
        for (int e = nsurv + tid; e < npad; e += nt) surv[e] = ~0ull;
        if (npad <= 4 * nt) block_sort_lds<4>(surv, npad, tid, nt);
        else bitonic_sort_lds(surv, npad, tid, nt);            // more than four keys per thread: all in LDS
        for (int e = tid; e < kk; e += nt) {
            const unsigned long long skey = surv[e];
            g.out_ids[(size_t)q * k + e] = (int64_t)(uint32_t)skey;
            g.out_dists[(size_t)q * k + e] = mono_inv((uint32_t)(skey >> 32));
        }
    }
    for (int e = kk + tid; e < k; e += nt) {
        g.out_ids[(size_t)q * k + e] = (int64_t)-1;
        g.out_dists[(size_t)q * k + e] = __builtin_inff();
    }
}


// ---- one translation unit per code width instantiates its kernels through these ------------------------------
// HAS_TAPS: a variant with the taps exists for this code width (the word-wise (pair, lambda) variants have none:
// the tapped call takes the byte-wise kernel).
template <int MW, bool HAS_TAPS>
inline hipError_t launch_rerank_variant(const RerankArgs& a, const RerankLds& L, const RankArgs& rk, const RankOffsets& RL,
                                        bool taps, bool fused, hipStream_t s) {
    const dim3 grid((unsigned)(a.nq + a.early)), block(a.threads);
    if (fused) {
        hipLaunchKernelGGL((rerank_kernel<MW, false, true>), grid, block, L.total, s, a, L, rk, RL);
    } else if (taps) {
        if constexpr (HAS_TAPS) hipLaunchKernelGGL((rerank_kernel<MW, true, false>), grid, block, L.total, s, a, L, rk, RL);
        else return hipErrorInvalidValue;
    } else {
        hipLaunchKernelGGL((rerank_kernel<MW, false, false>), grid, block, L.total, s, a, L, rk, RL);
    }
    return hipGetLastError();
}

template <int MW, bool HAS_TAPS>
inline hipError_t configure_rerank_variant(size_t max_dynamic_lds) {
    const void* kernels[3] = {reinterpret_cast<const void*>(rerank_kernel<MW, false, false>),
                              reinterpret_cast<const void*>(rerank_kernel<MW, false, true>), nullptr};
    if constexpr (HAS_TAPS) kernels[2] = reinterpret_cast<const void*>(rerank_kernel<MW, true, false>);
    for (const void* kfn : kernels) {
        if (!kfn) continue;
        hipFuncAttributes attr;
        hipError_t e = hipFuncGetAttributes(&attr, kfn);
        if (e != hipSuccess) return e;
        if (attr.sharedSizeBytes != 0) return hipErrorInvalidValue;   // the LUT must start at LDS address 0
        e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

#define PQT_RERANK_VARIANT_DEFINE(NAME, MW, HAS_TAPS)                                                                       \
    hipError_t launch_rerank_##NAME(const RerankArgs& a, const RerankLds& L, const RankArgs& rk, const RankOffsets& RL,      \
                                    bool taps, bool fused, hipStream_t s) {                                                 \
        return launch_rerank_variant<MW, HAS_TAPS>(a, L, rk, RL, taps, fused, s);                                           \
    }                                                                                                                       \
    hipError_t configure_rerank_##NAME(size_t max_dynamic_lds) { return configure_rerank_variant<MW, HAS_TAPS>(max_dynamic_lds); }

}  // namespace pqt
