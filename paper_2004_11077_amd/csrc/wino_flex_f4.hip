// Flex kernels for F(4x4, 3x3).
#include "wino_flex.hpp"

namespace wino {
template struct PerMFlex<4>;
}  // namespace wino
