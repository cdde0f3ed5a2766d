// Instantiates the contraction + output-transform kernels of F(6 x 6, 3 x 3).
#include "wino_conout.hpp"

namespace wino {
template struct PerMCO<6>;
}
