// The small-state step kernel and its Eq. 8 kernel for k = 16, d = 8.
#include "small_steps.h"

namespace asgd {

ASGD_SMALL_SHAPE_DEFINE(16, 8, false)

}  // namespace asgd
