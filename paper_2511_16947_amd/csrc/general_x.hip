// Replica loads for a restricted placement (Eq. 1 with G_EDP^e a strict subset).
#include "common.h"

namespace fine {

int launch_general_x(const fine_shape& s, const uint8_t* place, const int32_t* load, int32_t* x_eg,
                     int32_t* max_load, int32_t* scratch, hipStream_t st) {
    (void)s; (void)place; (void)load; (void)x_eg; (void)max_load; (void)scratch; (void)st;
    return FINE_UNSUPPORTED;
}

}  // namespace fine
