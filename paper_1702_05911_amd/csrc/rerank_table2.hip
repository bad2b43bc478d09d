// The re-rank kernel for one-byte codes, M = 8.
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(table2, 2, true)
}  // namespace pqt
