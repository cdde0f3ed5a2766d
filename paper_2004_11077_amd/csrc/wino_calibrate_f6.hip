// Instantiates the calibration kernels of F(6 x 6, 3 x 3).
#include "wino_calibrate.hpp"

namespace wino {
template struct PerMCal<6>;
}
