// The re-rank kernel for (pair, lambda) codes, M = 8.
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(pair8, -8, false)
}  // namespace pqt
