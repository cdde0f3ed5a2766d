// Instantiates the transform kernels of F(2 x 2, 3 x 3).
#include "wino_transforms.hpp"

namespace wino {
template struct PerM<2>;
}
