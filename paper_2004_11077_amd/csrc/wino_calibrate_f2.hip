// Instantiates the calibration kernels of F(2 x 2, 3 x 3).
#include "wino_calibrate.hpp"

namespace wino {
template struct PerMCal<2>;
}
