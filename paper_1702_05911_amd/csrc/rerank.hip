// Vector proposal, re-ranking by line quantisation and the final ordering
// (Sec. 3.2 "vector proposal", Sec. 3.3 "Online computation" Eq. 8-9, Sec. 4 last kernel).
//
// One workgroup per query.
//   * the per-query table LUT[m][c] of Eq. 9 summands is built in LDS from the level-1
//     sub-part distances the traversal already produced (no new distance is computed);
//   * codes are stored bin-major beside the ids, so the candidates of a proposed slot are one
//     contiguous run: lanes walk candidate positions, consecutive lanes read consecutive
//     codes (coalesced); the run of a position is found by a short binary search over the run
//     starts held in LDS; the id array is only touched for the few survivors;
//   * score = sum over m = 0..M-1, in that order, of LUT[m][code[m]] in fp32;
//   * the k best by (score, id): one histogram over the ordered score bits between the smallest
//     and largest score of the query finds a bucket b that holds the k-th smallest; everything
//     in buckets <= b (a superset of the answer, normally a few more than k) is collected as
//     64-bit keys (score bits, id) and ordered by counting ranks.  If the superset does not fit
//     (heavily tied scores) an exact radix select on score bits, then on ids, picks exactly k.
#include "pqt_device.hpp"
#include "pqt_kernels.hpp"

namespace pqt {

constexpr int kHistBits = 11;
constexpr int kHistSize = 1 << kHistBits;
constexpr int kCountRankMax = 512;   // survivors ordered by counting ranks up to this many, else bitonic

struct RerankLds {
    int kpad, scap;
    uint32_t surv, lut, a, run_src, run_start, skey, hist, part, misc, total;
};

static RerankLds rerank_layout(int M, int k1, int T, int C, int k, int threads) {
    RerankLds L;
    L.kpad = next_pow2(k);
    L.scap = 2 * L.kpad < 256 ? 256 : 2 * L.kpad;
    size_t o = 0;
    L.surv = (uint32_t)o;      o += sizeof(unsigned long long) * L.scap;
    L.lut = (uint32_t)o;       o += sizeof(float) * M * 256;
    L.a = (uint32_t)o;         o += sizeof(float) * M * k1;
    L.run_src = (uint32_t)o;   o += sizeof(uint32_t) * T;
    L.run_start = (uint32_t)o; o += sizeof(uint32_t) * (T + 1);
    L.skey = (uint32_t)o;      o += sizeof(uint32_t) * C;
    L.hist = (uint32_t)o;      o += sizeof(uint32_t) * kHistSize;
    L.part = (uint32_t)o;      o += sizeof(uint32_t) * threads;
    L.misc = (uint32_t)o;      o += sizeof(uint32_t) * 16;
    o = (o + 15) & ~size_t(15);
    L.total = (uint32_t)o;
    return L;
}

size_t rerank_lds_bytes(int M, int k1, int T, int C, int k, int threads) {
    return rerank_layout(M, k1, T, C, k, threads).total;
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

__device__ __forceinline__ uint32_t wave_sum_inclusive(uint32_t v, int lane) {
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t n = __shfl_up(v, off, kWave);
        if (lane >= off) v += n;
    }
    return v;
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
enum { kMin = 0, kMax = 1, kBucket = 2, kCountLe = 3, kNumSurv = 4, kRadix = 8 };

// MW = 32-bit words per code (M/4) for M in {4, 8, 16, 32}; 0 = any other M (byte loads).
template <int MW>
__global__ __launch_bounds__(1024) void rerank_kernel(RerankArgs g, RerankLds L) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* surv = reinterpret_cast<unsigned long long*>(smem + L.surv);
    float* lut = reinterpret_cast<float*>(smem + L.lut);
    float* sa = reinterpret_cast<float*>(smem + L.a);
    uint32_t* run_src = reinterpret_cast<uint32_t*>(smem + L.run_src);
    uint32_t* run_start = reinterpret_cast<uint32_t*>(smem + L.run_start);
    uint32_t* skey = reinterpret_cast<uint32_t*>(smem + L.skey);
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
    uint32_t* part = reinterpret_cast<uint32_t*>(smem + L.part);
    uint32_t* misc = reinterpret_cast<uint32_t*>(smem + L.misc);

    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int64_t q = blockIdx.x;
    const int M = g.M, k1 = g.k1, T = g.T, C = g.C, k = g.k;
    const uint2 meta = g.meta[q];
    const int nr = (int)meta.x;
    const int nc = (int)meta.y;
    int steps = 0;
    while ((1 << steps) < nr) ++steps;

    // ---- run list and level-1 distances into LDS ---------------------------------------------------
    for (int r = tid; r < nr; r += nt) {
        const uint2 run = g.runs[(size_t)q * T + r];
        run_src[r] = run.x;
        run_start[r] = run.y;
    }
    if (tid == 0) {
        run_start[nr] = (uint32_t)nc;
        misc[kMin] = 0xffffffffu;
        misc[kMax] = 0u;
        misc[kNumSurv] = 0u;
    }
    for (int e = tid; e < M * k1; e += nt) sa[e] = g.a[(size_t)q * M * k1 + e];
    for (int e = tid; e < kHistSize; e += nt) hist[e] = 0;
    __syncthreads();

    // ---- LUT of Eq. 9 summands: b^2 + lam^2 c^2 + lam (a^2 - b^2 - c^2) ----------------------------
    for (int base = 0; base < M * 256; base += nt * 4) {
        CodeEntry ent[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = base + u * nt + tid;
            ent[u] = g.table[e < M * 256 ? e : 0];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = base + u * nt + tid;
            if (e >= M * 256) continue;
            const int m = e >> 8;
            const float b2 = sa[m * k1 + (ent[u].ij & 0xffu)];
            const float a2 = sa[m * k1 + ((ent[u].ij >> 8) & 0xffu)];
            const float v = (b2 + (ent[u].lam * ent[u].lam) * ent[u].cc) + ent[u].lam * ((a2 - b2) - ent[u].cc);
            lut[e] = v;
            if (g.lut) g.lut[(size_t)q * M * 256 + e] = v;
        }
    }
    __syncthreads();

    // ---- scores: kUnroll candidate positions per thread in flight (code loads issued before use) ----
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    constexpr int kUnroll = 4;
    for (int base = 0; base < nc; base += nt * kUnroll) {
        uint32_t src[kUnroll];
        uint32_t cw[kUnroll][MW > 0 ? MW : 1];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int p = base + u * nt + tid;
            src[u] = (p < nc) ? source_of((uint32_t)p, nr, steps, run_src, run_start) : run_src[0];
        }
        if (MW > 0) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const uint32_t* c = reinterpret_cast<const uint32_t*>(g.codes + (size_t)src[u] * M);
                if (MW == 2) {
                    const uint2 v = *reinterpret_cast<const uint2*>(c);
                    cw[u][0] = v.x;
                    cw[u][MW > 1 ? 1 : 0] = v.y;
                } else if (MW == 4) {
                    const uint4 v = *reinterpret_cast<const uint4*>(c);
                    cw[u][0] = v.x;
                    cw[u][MW > 1 ? 1 : 0] = v.y;
                    cw[u][MW > 2 ? 2 : 0] = v.z;
                    cw[u][MW > 3 ? 3 : 0] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < MW; ++j) cw[u][j] = c[j];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int p = base + u * nt + tid;
            if (p >= nc) continue;
            float s = 0.0f;
            if (MW > 0) {
#pragma unroll
                for (int j = 0; j < MW; ++j) {
                    const uint32_t wv = cw[u][j];
                    s += lut[(j * 4 + 0) * 256 + (wv & 0xffu)];
                    s += lut[(j * 4 + 1) * 256 + ((wv >> 8) & 0xffu)];
                    s += lut[(j * 4 + 2) * 256 + ((wv >> 16) & 0xffu)];
                    s += lut[(j * 4 + 3) * 256 + (wv >> 24)];
                }
            } else {
                const uint8_t* code = g.codes + (size_t)src[u] * M;
                for (int m = 0; m < M; ++m) s += lut[m * 256 + code[m]];
            }
            const uint32_t key = mono_key(s);
            skey[p] = key;
            kmin = min(kmin, key);
            kmax = max(kmax, key);
            if (g.scores) g.scores[(size_t)q * C + p] = s;
            if (g.cand_ids) g.cand_ids[(size_t)q * C + p] = (int64_t)g.ids[src[u]];
        }
    }
    if (g.n_cand && tid == 0) g.n_cand[q] = (uint32_t)nc;
    for (int off = kWave / 2; off > 0; off >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off, kWave));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off, kWave));
    }
    if (lane == 0) {
        atomicMin(&misc[kMin], kmin);
        atomicMax(&misc[kMax], kmax);
    }
    __syncthreads();

    // ---- the k smallest (score, id) --------------------------------------------------------------------
    const int kk = k < nc ? k : nc;           // results that exist
    int nsurv;
    if (nc <= L.scap) {                        // few candidates: order all of them
        for (int p = tid; p < nc; p += nt)
            surv[p] = ((unsigned long long)skey[p] << 32) | g.ids[source_of((uint32_t)p, nr, steps, run_src, run_start)];
        nsurv = nc;
    } else {
        const uint32_t lo_key = misc[kMin];
        const uint32_t range = misc[kMax] - lo_key;
        int shift = 0;
        while ((range >> shift) >= (uint32_t)kHistSize) ++shift;
        for (int p = tid; p < nc; p += nt) atomicAdd(&hist[(skey[p] - lo_key) >> shift], 1u);
        __syncthreads();
        // bucket b with count(< b) < kk <= count(<= b)
        {
            const int cb = kHistSize / nt;                       // bins per thread (nt divides 2048)
            uint32_t s = 0;
            for (int j = 0; j < cb; ++j) s += hist[tid * cb + ((j + (lane >> 2)) & (cb - 1))];
            part[tid] = s;
        }
        __syncthreads();
        if (tid < kWave) {
            const int pl = nt / kWave;                           // partial sums per lane
            uint32_t ls = 0;
            for (int i = 0; i < pl; ++i) ls += part[lane * pl + i];
            const uint32_t incl = wave_sum_inclusive(ls, lane);
            uint32_t c = incl - ls;
            if (c < (uint32_t)kk && (uint32_t)kk <= incl) {      // exactly one lane
                const int cb = kHistSize / nt;
                int i = lane * pl;
                while (c + part[i] < (uint32_t)kk) c += part[i++];
                int b = i * cb;
                while (c + hist[b] < (uint32_t)kk) c += hist[b++];
                misc[kBucket] = (uint32_t)b;
                misc[kCountLe] = c + hist[b];
            }
        }
        __syncthreads();
        const uint32_t b = misc[kBucket];
        const uint32_t count_le = misc[kCountLe];
        if (count_le <= (uint32_t)L.scap) {
            for (int p = tid; p < nc; p += nt) {
                const uint32_t key = skey[p];
                if (((key - lo_key) >> shift) <= b) {
                    const uint32_t id = g.ids[source_of((uint32_t)p, nr, steps, run_src, run_start)];
                    surv[atomicAdd(&misc[kNumSurv], 1u)] = ((unsigned long long)key << 32) | id;
                }
            }
            nsurv = (int)count_le;
        } else {
            // exact selection: k-th smallest score key, then (only if that score is tied) the ids
            uint32_t* rout = misc + kRadix;
            uint32_t prefix = 0, mask = 0, need = (uint32_t)kk, bucket = 0;
            const int shifts[3] = {21, 10, 0};
            const int nbits[3] = {11, 11, 10};
            for (int pass = 0; pass < 3; ++pass) {
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
                for (int pass = 0; pass < 3; ++pass) {
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
                const uint32_t id = g.ids[source_of((uint32_t)p, nr, steps, run_src, run_start)];
                if (key == tau && id > id_cut) continue;
                surv[atomicAdd(&misc[kNumSurv], 1u)] = ((unsigned long long)key << 32) | id;
            }
            nsurv = kk;
        }
    }
    __syncthreads();

    // ---- order the survivors, write the first k ---------------------------------------------------------
    if (nsurv <= kCountRankMax) {
        for (int e = tid; e < nsurv; e += nt) {
            const unsigned long long key = surv[e];
            int rank = 0;
            for (int j = 0; j < nsurv; ++j) rank += (surv[j] < key) ? 1 : 0;
            if (rank < k) {
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

hipError_t launch_rerank(const RerankArgs& a, hipStream_t s) {
    if (a.nq <= 0) return hipSuccess;
    const RerankLds L = rerank_layout(a.M, a.k1, a.T, a.C, a.k, a.threads);
    const dim3 grid((unsigned)a.nq), block(a.threads);
    switch ((a.M % 4 == 0) ? a.M / 4 : 0) {
        case 1: hipLaunchKernelGGL(rerank_kernel<1>, grid, block, L.total, s, a, L); break;
        case 2: hipLaunchKernelGGL(rerank_kernel<2>, grid, block, L.total, s, a, L); break;
        case 4: hipLaunchKernelGGL(rerank_kernel<4>, grid, block, L.total, s, a, L); break;
        case 8: hipLaunchKernelGGL(rerank_kernel<8>, grid, block, L.total, s, a, L); break;
        default: hipLaunchKernelGGL(rerank_kernel<0>, grid, block, L.total, s, a, L); break;
    }
    return hipGetLastError();
}

hipError_t configure_rerank(size_t max_dynamic_lds) {
    const void* kernels[] = {reinterpret_cast<const void*>(rerank_kernel<0>), reinterpret_cast<const void*>(rerank_kernel<1>),
                             reinterpret_cast<const void*>(rerank_kernel<2>), reinterpret_cast<const void*>(rerank_kernel<4>),
                             reinterpret_cast<const void*>(rerank_kernel<8>)};
    for (const void* kfn : kernels) {
        hipError_t e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace pqt
