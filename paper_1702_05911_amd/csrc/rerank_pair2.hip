// The re-rank kernel for (pair, lambda) codes, M = 2.
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(pair2, -2, false)
}  // namespace pqt
