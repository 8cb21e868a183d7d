// Explicit instantiation of the small-policy whole-network kernel with one row tile per workgroup, in the form
// for a workgroup that has its CU to itself (per-channel symmetric weights), with and without intermediate taps.
#include "rows16_mlp.hpp"

namespace aq {
namespace r16 {
AQ_ROWS16_LATE_INST(false);
}  // namespace r16
}  // namespace aq
