// Explicit instantiation of one fused-MLP kernel variant (16 rows per workgroup, per-tensor asymmetric
// weights), with and without intermediate taps.
#include "fused_mlp.hpp"

namespace aq {
AQ_FUSED_INST(1, 1, true, false, true);
AQ_FUSED_INST(1, 1, true, true, true);
}  // namespace aq
