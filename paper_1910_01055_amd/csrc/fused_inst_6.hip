// Explicit instantiation of one fused-MLP kernel variant (rows = 32 * 2, 1 feature tile(s) per wave,
// per-tensor asymmetric weights), with and without intermediate taps.
#include "fused_mlp.hpp"

namespace aq {
AQ_FUSED_INST(2, 1, true, false, false);
AQ_FUSED_INST(2, 1, true, true, false);
}  // namespace aq
