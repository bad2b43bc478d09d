// The re-rank kernel for one-byte codes of any length (byte loads).
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(table0, 0, true)
}  // namespace pqt
