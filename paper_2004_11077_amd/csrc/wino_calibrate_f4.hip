// Instantiates the calibration kernels of F(4 x 4, 3 x 3).
#include "wino_calibrate.hpp"

namespace wino {
template struct PerMCal<4>;
}
