// Vector proposal, re-ranking by line quantisation and the final ordering
// (Sec. 3.2 "vector proposal", Sec. 3.3 "Online computation" Eq. 8-9, Sec. 4 last kernel).
//
// One workgroup per query.
//   * the per-query table LUT[m][c] of Eq. 9 summands is built in LDS from the level-1
//     sub-part distances the traversal already produced (no new distance is computed);
//   * codes are stored bin-major beside the ids, so the candidates of a proposed slot are one
//     contiguous run: lanes walk candidate positions, consecutive lanes read consecutive
//     codes (coalesced) -- the id array is only touched for the few survivors;
//   * score = sum over m = 0..M-1, in that order, of LUT[m][code[m]] in fp32;
//   * the k best by (score, id) are found by a radix select on the ordered score bits
//     (and, only if the k-th score is tied, on the ids of the tied candidates), then the
//     <= k survivors are sorted as 64-bit keys.
#include "pqt_device.hpp"
#include "pqt_kernels.hpp"

namespace pqt {

constexpr int kHistBits = 11;
constexpr int kHistSize = 1 << kHistBits;

struct RerankLds {
    int kpad;
    uint32_t lut, a, run_src, run_start, runidx, skey, hist, surv, part, misc, total;
};

static RerankLds rerank_layout(int M, int k1, int T, int C, int k, int threads) {
    RerankLds L;
    L.kpad = next_pow2(k);
    size_t o = 0;
    L.surv = (uint32_t)o;      o += sizeof(unsigned long long) * L.kpad;
    L.lut = (uint32_t)o;       o += sizeof(float) * M * 256;
    L.a = (uint32_t)o;         o += sizeof(float) * M * k1;
    L.run_src = (uint32_t)o;   o += sizeof(uint32_t) * T;
    L.run_start = (uint32_t)o; o += sizeof(uint32_t) * (T + 1);
    L.skey = (uint32_t)o;      o += sizeof(uint32_t) * C;
    L.hist = (uint32_t)o;      o += sizeof(uint32_t) * kHistSize;
    L.part = (uint32_t)o;      o += sizeof(uint32_t) * threads;
    L.misc = (uint32_t)o;      o += sizeof(uint32_t) * 8;
    L.runidx = (uint32_t)o;    o += sizeof(uint16_t) * C;
    o = (o + 15) & ~size_t(15);
    L.total = (uint32_t)o;
    return L;
}

size_t rerank_lds_bytes(int M, int k1, int T, int C, int k, int threads) {
    return rerank_layout(M, k1, T, C, k, threads).total;
}

// Position p of the candidate list -> position in ids/codes.
__device__ __forceinline__ uint32_t source_of(int p, const uint16_t* runidx, const uint32_t* run_src,
                                              const uint32_t* run_start) {
    const uint32_t r = runidx[p];
    return run_src[r] + ((uint32_t)p - run_start[r]);
}

// One pass of a most-significant-digit radix select.  Counts, among the n items whose key
// agrees with `prefix` on the bits of `mask`, the digit (key >> shift) & (2^bits - 1); finds
// the digit holding the item of 1-based rank *need, updates *need to the rank inside it.
// get_key(p, &valid) supplies the keys.  misc[0] = digit, misc[1] = new need, misc[2] = size
// of the chosen digit's bucket.  All threads must call it; ends with a barrier.
template <typename KeyFn>
__device__ __forceinline__ void radix_select_pass(int n, uint32_t prefix, uint32_t mask, int shift, int bits,
                                                  uint32_t need, uint32_t* hist, uint32_t* part,
                                                  uint32_t* misc, KeyFn get_key) {
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
    // keep the counts: the scan works on a copy held in registers per thread chunk
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
            misc[0] = (uint32_t)e;
            misc[1] = need - s;
            misc[2] = c;
        }
        s += c;
    }
    __syncthreads();
}

__global__ __launch_bounds__(1024) void rerank_kernel(RerankArgs g, RerankLds L) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* surv = reinterpret_cast<unsigned long long*>(smem + L.surv);
    float* lut = reinterpret_cast<float*>(smem + L.lut);
    float* sa = reinterpret_cast<float*>(smem + L.a);
    uint32_t* run_src = reinterpret_cast<uint32_t*>(smem + L.run_src);
    uint32_t* run_start = reinterpret_cast<uint32_t*>(smem + L.run_start);
    uint16_t* runidx = reinterpret_cast<uint16_t*>(smem + L.runidx);
    uint32_t* skey = reinterpret_cast<uint32_t*>(smem + L.skey);
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
    uint32_t* part = reinterpret_cast<uint32_t*>(smem + L.part);
    uint32_t* misc = reinterpret_cast<uint32_t*>(smem + L.misc);

    const int tid = threadIdx.x, nt = blockDim.x;
    const int64_t q = blockIdx.x;
    const int M = g.M, k1 = g.k1, T = g.T, C = g.C, k = g.k;
    const uint2 meta = g.meta[q];
    const int nr = (int)meta.x;
    const int nc = (int)meta.y;

    // ---- run list and level-1 distances into LDS ---------------------------------------------------
    for (int r = tid; r < nr; r += nt) {
        const uint2 run = g.runs[(size_t)q * T + r];
        run_src[r] = run.x;
        run_start[r] = run.y;
    }
    if (tid == 0) run_start[nr] = (uint32_t)nc;
    for (int e = tid; e < M * k1; e += nt) sa[e] = g.a[(size_t)q * M * k1 + e];
    for (int p = tid; p < nc; p += nt) runidx[p] = 0;
    __syncthreads();

    // ---- LUT of Eq. 9 summands: b^2 + lam^2 c^2 + lam (a^2 - b^2 - c^2) ----------------------------
    for (int e = tid; e < M * 256; e += nt) {
        const CodeEntry ent = g.table[e];
        const int m = e >> 8;
        const float b2 = sa[m * k1 + (ent.ij & 0xffu)];
        const float a2 = sa[m * k1 + ((ent.ij >> 8) & 0xffu)];
        const float v = (b2 + (ent.lam * ent.lam) * ent.cc) + ent.lam * ((a2 - b2) - ent.cc);
        lut[e] = v;
        if (g.lut) g.lut[(size_t)q * M * 256 + e] = v;
    }
    // ---- candidate position -> run: mark run heads, running maximum --------------------------------
    for (int r = tid + 1; r < nr; r += nt) runidx[run_start[r]] = (uint16_t)r;
    __syncthreads();
    block_inclusive_max_u16(runidx, nc, part);

    // ---- scores --------------------------------------------------------------------------------------
    for (int p = tid; p < nc; p += nt) {
        const uint32_t src = source_of(p, runidx, run_src, run_start);
        const uint8_t* code = g.codes + (size_t)src * M;
        float s = 0.0f;
        if ((M & 3) == 0) {
            const uint32_t* cw = reinterpret_cast<const uint32_t*>(code);
            for (int m4 = 0; m4 < M / 4; ++m4) {
                const uint32_t wv = cw[m4];
                s += lut[(m4 * 4 + 0) * 256 + (wv & 0xffu)];
                s += lut[(m4 * 4 + 1) * 256 + ((wv >> 8) & 0xffu)];
                s += lut[(m4 * 4 + 2) * 256 + ((wv >> 16) & 0xffu)];
                s += lut[(m4 * 4 + 3) * 256 + (wv >> 24)];
            }
        } else {
            for (int m = 0; m < M; ++m) s += lut[m * 256 + code[m]];
        }
        skey[p] = mono_key(s);
        if (g.scores) g.scores[(size_t)q * C + p] = s;
        if (g.cand_ids) g.cand_ids[(size_t)q * C + p] = (int64_t)g.ids[src];
    }
    if (g.n_cand && tid == 0) g.n_cand[q] = (uint32_t)nc;
    __syncthreads();

    // ---- the k smallest (score, id) --------------------------------------------------------------------
    const int kk = k < nc ? k : nc;          // results that exist
    uint32_t tau = 0xffffffffu;               // k-th smallest score key
    uint32_t id_cut = 0xffffffffu;            // among candidates with key == tau keep ids <= id_cut
    if (nc > k) {
        uint32_t prefix = 0, mask = 0, need = (uint32_t)kk;
        const int shifts[3] = {21, 10, 0};
        const int nbits[3] = {11, 11, 10};
        uint32_t bucket = 0;
        for (int pass = 0; pass < 3; ++pass) {
            radix_select_pass(nc, prefix, mask, shifts[pass], nbits[pass], need, hist, part, misc,
                              [&](int p, bool& valid) { valid = true; return skey[p]; });
            prefix |= misc[0] << shifts[pass];
            mask |= ((1u << nbits[pass]) - 1u) << shifts[pass];
            need = misc[1];
            bucket = misc[2];
            __syncthreads();
        }
        tau = prefix;
        if (need < bucket) {                  // the k-th score is tied: take the `need` smallest ids
            uint32_t iprefix = 0, imask = 0;
            for (int pass = 0; pass < 3; ++pass) {
                radix_select_pass(nc, iprefix, imask, shifts[pass], nbits[pass], need, hist, part, misc,
                                  [&](int p, bool& valid) {
                                      valid = skey[p] == tau;
                                      return valid ? g.ids[source_of(p, runidx, run_src, run_start)] : 0u;
                                  });
                iprefix |= misc[0] << shifts[pass];
                imask |= ((1u << nbits[pass]) - 1u) << shifts[pass];
                need = misc[1];
                __syncthreads();
            }
            id_cut = iprefix;
        }
    }
    for (int e = tid; e < L.kpad; e += nt) surv[e] = ~0ull;
    if (tid == 0) misc[4] = 0;
    __syncthreads();
    for (int p = tid; p < nc; p += nt) {
        const uint32_t key = skey[p];
        if (key > tau) continue;
        const uint32_t id = g.ids[source_of(p, runidx, run_src, run_start)];
        if (key == tau && id > id_cut) continue;
        const uint32_t at = atomicAdd(&misc[4], 1u);
        if (at < (uint32_t)L.kpad) surv[at] = ((unsigned long long)key << 32) | id;
    }
    bitonic_sort_lds(surv, L.kpad, tid, nt);
    for (int e = tid; e < k; e += nt) {
        const unsigned long long key = surv[e];
        const bool have = e < kk;
        g.out_ids[(size_t)q * k + e] = have ? (int64_t)(uint32_t)key : (int64_t)-1;
        g.out_dists[(size_t)q * k + e] = have ? mono_inv((uint32_t)(key >> 32)) : __builtin_inff();
    }
}

hipError_t launch_rerank(const RerankArgs& a, hipStream_t s) {
    if (a.nq <= 0) return hipSuccess;
    const RerankLds L = rerank_layout(a.M, a.k1, a.T, a.C, a.k, a.threads);
    hipLaunchKernelGGL(rerank_kernel, dim3((unsigned)a.nq), dim3(a.threads), L.total, s, a, L);
    return hipGetLastError();
}

hipError_t configure_rerank(size_t max_dynamic_lds) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(rerank_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
}

}  // namespace pqt
