// Instantiates the transform kernels of F(6 x 6, 3 x 3).
#include "wino_transforms.hpp"

namespace wino {
template struct PerM<6>;
}
