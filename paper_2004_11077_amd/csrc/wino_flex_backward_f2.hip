// Flex backward kernels of F(2x2, 3x3).
#include "wino_flex_backward.hpp"
namespace wino {
template struct PerMFlexBwd<2>;
}  // namespace wino
