// The re-rank kernel for one-byte codes, M = 4.
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(table1, 1, true)
}  // namespace pqt
