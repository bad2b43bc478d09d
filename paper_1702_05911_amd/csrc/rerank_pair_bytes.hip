// The re-rank kernel for (pair, lambda) codes of any length (byte loads).
#include "rerank_kernel.hpp"

namespace pqt {
PQT_RERANK_VARIANT_DEFINE(pair_bytes, kPairLambda, true)
}  // namespace pqt
