// Host side of the re-rank stage (Sec. 3.2 "vector proposal", Sec. 3.3 "Online computation" Eq. 8-9, Sec. 4
// last kernel): LDS layout, workgroup shape, and the dispatch to the kernel variant for the index's code
// width.  The kernel itself is in rerank_kernel.hpp, compiled per code width in rerank_table*.hip and
// rerank_pair*.hip.
#include "pqt_device.hpp"
#include "rank_head_device.hpp"
#include "rerank_variants.hpp"

namespace pqt {

static RerankLds rerank_layout(int M, int k1, int T, int C, int k, int threads, size_t rank_lds, int code_format,
                               int runs_in_lds) {
    RerankLds L;
    (void)C;
    L.kpad = next_pow2(k);
    L.scap = 2 * L.kpad < 256 ? 256 : 2 * L.kpad;
    const int want = runs_in_lds < kRunsInLdsMin ? kRunsInLdsMin : runs_in_lds;
    L.rcap = T < want ? T : want;
    size_t o = 0;
    // at offset 0: lookups need no base register.
    // One float per table entry, or (b^2, a^2 - b^2, c^2, -) per centroid pair for (pair, lambda) codes.
    L.lut = (uint32_t)o;       o += code_format == 1 ? sizeof(float4) * ((size_t)M << pair_table_shift(k1)) : sizeof(float) * M * 256;
    L.surv = (uint32_t)o;      o += sizeof(unsigned long long) * L.scap;
    L.hist = (uint32_t)o;      o += sizeof(uint32_t) * kHistSize;
    L.part = (uint32_t)o;      o += sizeof(uint32_t) * threads;      // scan scratch of the exact selection
    // everything above is free while a workgroup runs the full bin ranking of its query, which uses
    // the first rank_lds bytes; the arrays below receive its result
    if (o < rank_lds) o = (rank_lds + 15) & ~size_t(15);
    L.a = (uint32_t)o;         o += sizeof(float) * M * k1;
    L.run_src = (uint32_t)o;   o += sizeof(uint32_t) * L.rcap;
    L.run_start = (uint32_t)o; o += sizeof(uint32_t) * (L.rcap + 1);
    L.misc = (uint32_t)o;      o += sizeof(uint32_t) * 16;
    o = (o + 15) & ~size_t(15);
    L.total = (uint32_t)o;
    return L;
}

size_t rerank_lds_bytes(int M, int k1, int T, int C, int k, int threads, size_t rank_lds, int code_format,
                        int runs_in_lds) {
    return rerank_layout(M, k1, T, C, k, threads, rank_lds, code_format, runs_in_lds).total;
}

void rerank_shape(int C, int M, int code_format, int* threads, int* keys_per_thread) {
    int t = 256;
    while (t < 1024 && C > kKeysPerThread * t) t *= 2;
    (void)M;
    (void)code_format;
    *threads = t;
    *keys_per_thread = kKeysPerThread;
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
        RL = rank_offsets(rk.P, rk.R, rk.T, rk.hashed, false);
        if (RL.Tcap > rerank_fused_tuples_per_thread() * a.threads) return hipErrorInvalidValue;
        // the wavefront's two lists lie at the start of the workgroup's LDS (table, survivor list and
        // histogram are not in use yet, and the arrays that receive the result come after them)
        static_assert(sizeof(HeadLds) <= sizeof(uint32_t) * kHistSize, "the lists must end before the arrays that are live");
        a.mid_T1 = RL.Tcap < kHeadT ? RL.Tcap : kHeadT;
        a.mid_npairs = head_pair_count(a.mid_T1);
    }
    if (a.keys_per_thread != kKeysPerThread || a.C > a.keys_per_thread * a.threads) return hipErrorInvalidValue;
    if (a.threads % 256 != 0) return hipErrorInvalidValue;             // a thread builds the table entries of one code value
    if (a.code_format == 1 && a.lut) return hipErrorInvalidValue;      // that tap is the one-byte format's table
    const RerankLds L = rerank_layout(a.M, a.k1, a.T, a.C, a.k, a.threads, fused ? RL.total : 0, a.code_format, a.runs_in_lds);
    const bool f = fused != nullptr;
    if (a.code_format == 1) {
        // word-wise variants for the plain entry point; the tapped one takes the byte-wise kernel
        switch (taps || a.M % 2 ? 0 : a.M / 2) {
            case 2: return launch_rerank_pair2(a, L, rk, RL, taps, f, s);
            case 4: return launch_rerank_pair4(a, L, rk, RL, taps, f, s);
            case 8: return launch_rerank_pair8(a, L, rk, RL, taps, f, s);
            default: return launch_rerank_pair_bytes(a, L, rk, RL, taps, f, s);
        }
    }
    switch ((a.M % 4 == 0) ? a.M / 4 : 0) {
        case 1: return launch_rerank_table1(a, L, rk, RL, taps, f, s);
        case 2: return launch_rerank_table2(a, L, rk, RL, taps, f, s);
        case 4: return launch_rerank_table4(a, L, rk, RL, taps, f, s);
        case 8: return launch_rerank_table8(a, L, rk, RL, taps, f, s);
        default: return launch_rerank_table0(a, L, rk, RL, taps, f, s);
    }
}

hipError_t configure_rerank(size_t max_dynamic_lds) {
    hipError_t (*const all[])(size_t) = {configure_rerank_table0, configure_rerank_table1, configure_rerank_table2,
                                         configure_rerank_table4, configure_rerank_table8, configure_rerank_pair_bytes,
                                         configure_rerank_pair2,  configure_rerank_pair4,  configure_rerank_pair8};
    for (auto fn : all) {
        const hipError_t e = fn(max_dynamic_lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace pqt
