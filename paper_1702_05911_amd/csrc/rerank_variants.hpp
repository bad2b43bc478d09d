// The re-rank kernel is compiled once per code width, each width in a translation unit of its own
// (rerank_table*.hip: one byte per sub-part, M = 4, 8, 16, 32 or any; rerank_pair*.hip: (pair, lambda)
// codes, M = 2, 4, 8 word-wise or any byte-wise).  This header declares their launchers.
#pragma once
#include "pqt_kernels.hpp"

namespace pqt {

struct RerankLds {
    int kpad, scap, rcap;
    uint32_t surv, lut, a, run_src, run_start, hist, part, misc, total;
};

#define PQT_RERANK_VARIANT_DECLARE(NAME)                                                                               \
    hipError_t launch_rerank_##NAME(const RerankArgs& a, const RerankLds& L, const RankArgs& rk, const RankOffsets& RL, \
                                    bool taps, bool fused, hipStream_t s);                                             \
    hipError_t configure_rerank_##NAME(size_t max_dynamic_lds);

PQT_RERANK_VARIANT_DECLARE(table0)
PQT_RERANK_VARIANT_DECLARE(table1)
PQT_RERANK_VARIANT_DECLARE(table2)
PQT_RERANK_VARIANT_DECLARE(table4)
PQT_RERANK_VARIANT_DECLARE(table8)
PQT_RERANK_VARIANT_DECLARE(pair_bytes)
PQT_RERANK_VARIANT_DECLARE(pair2)
PQT_RERANK_VARIANT_DECLARE(pair4)
PQT_RERANK_VARIANT_DECLARE(pair8)

// compile-time constants the host side needs as well
constexpr int kHistBits = 10;
constexpr int kHistSize = 1 << kHistBits;
constexpr int kFusedPer = 4;         // tuples per thread the in-kernel bin ranking may hold
constexpr int kKeysPerThread = 20;   // candidates a thread scores; C <= kKeysPerThread * workgroup size
constexpr int kRunsInLdsMin = 64;    // at least this many runs of a query are kept in LDS (see RerankArgs::runs_in_lds)

// (pair, lambda) codes: entries per sub-part in the LDS table of centroid pairs (128 while the pairs fit)
inline int pair_table_shift(int k1) { return k1 * (k1 - 1) / 2 <= 128 ? 7 : 8; }

}  // namespace pqt
