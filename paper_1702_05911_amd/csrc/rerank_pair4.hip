// The re-rank kernel for (pair, lambda) codes, M = 4.
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(pair4, -4, false)
}  // namespace pqt
