// Flex kernels for F(2x2, 3x3).
#include "wino_flex.hpp"

namespace wino {
template struct PerMFlex<2>;
}  // namespace wino
