// The small-state step kernel and its Eq. 8 kernel for k = 10, d = 10.
#include "small_steps.h"

namespace asgd {

ASGD_SMALL_SHAPE_DEFINE(10, 10, true)

}  // namespace asgd
