// Explicit instantiation of the small-policy whole-network kernel with 1 row tile(s) (16 batch rows) per
// workgroup for per-tensor asymmetric weights, with and without intermediate taps.
#include "rows16_mlp.hpp"

namespace aq {
namespace r16 {
AQ_ROWS16_INST(1, true);
}  // namespace r16
}  // namespace aq
