// Flex backward kernels of F(4x4, 3x3).
#include "wino_flex_backward.hpp"
namespace wino {
template struct PerMFlexBwd<4>;
}  // namespace wino
