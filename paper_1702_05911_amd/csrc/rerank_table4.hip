// The re-rank kernel for one-byte codes, M = 16.
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(table4, 4, true)
}  // namespace pqt
