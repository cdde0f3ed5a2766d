// Flex kernels for F(6x6, 3x3).
#include "wino_flex.hpp"

namespace wino {
template struct PerMFlex<6>;
}  // namespace wino
