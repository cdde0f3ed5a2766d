// Instantiates the transform kernels of F(4 x 4, 3 x 3).
#include "wino_transforms.hpp"

namespace wino {
template struct PerM<4>;
}
