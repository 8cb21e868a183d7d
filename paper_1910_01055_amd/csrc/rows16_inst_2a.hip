// Explicit instantiation of the small-policy whole-network kernel with 2 row tile(s) (32 batch rows) per
// workgroup for per-tensor asymmetric weights, with and without intermediate taps.
#include "rows16_mlp.hpp"

namespace aq {
namespace r16 {
AQ_ROWS16_INST(2, true);
}  // namespace r16
}  // namespace aq
