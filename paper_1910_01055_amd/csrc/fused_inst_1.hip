// Explicit instantiation of one fused-MLP kernel variant (rows = 32 * 2, 1 feature tile(s) per wave,
// symmetric weights), with and without intermediate taps.
#include "fused_mlp.hpp"

namespace aq {
AQ_FUSED_INST(2, 1, false, false, false);
AQ_FUSED_INST(2, 1, false, true, false);
}  // namespace aq
