// Flex backward kernels of F(6x6, 3x3).
#include "wino_flex_backward.hpp"
namespace wino {
template struct PerMFlexBwd<6>;
}  // namespace wino
