// Explicit instantiation of one fused-MLP kernel variant (16 rows per workgroup, symmetric weights),
// with and without intermediate taps.
#include "fused_mlp.hpp"

namespace aq {
AQ_FUSED_INST(1, 1, false, false, true);
AQ_FUSED_INST(1, 1, false, true, true);
}  // namespace aq
