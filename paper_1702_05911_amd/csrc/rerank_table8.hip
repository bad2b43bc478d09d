// The re-rank kernel for one-byte codes, M = 32.
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(table8, 8, true)
}  // namespace pqt
