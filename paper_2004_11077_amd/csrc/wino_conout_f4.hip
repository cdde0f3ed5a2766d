// Instantiates the contraction + output-transform kernels of F(4 x 4, 3 x 3).
#include "wino_conout.hpp"

namespace wino {
template struct PerMCO<4>;
}
