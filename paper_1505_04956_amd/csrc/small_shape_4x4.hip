// The small-state step kernel and its Eq. 8 kernel for k = 4, d = 4.
#include "small_steps.h"

namespace asgd {

ASGD_SMALL_SHAPE_DEFINE(4, 4, false)

}  // namespace asgd
