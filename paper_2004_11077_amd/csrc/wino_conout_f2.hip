// Instantiates the contraction + output-transform kernels of F(2 x 2, 3 x 3).
#include "wino_conout.hpp"

namespace wino {
template struct PerMCO<2>;
}
