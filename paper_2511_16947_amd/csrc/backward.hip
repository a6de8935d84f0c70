// Backward of permute + grouped FFN + combine.
#include "common.h"

namespace fine {

int launch_backward(const fine_shape& s, const void* d_out, const void* x_perm, const void* y_perm,
                    const void* act_save, const void* wg, const void* wu, const void* wd,
                    const int32_t* row_of_pair, const int32_t* pair_of_row, const int32_t* seg_off,
                    const float* topk_w, void* d_x, float* d_topk_w, float* d_wg, float* d_wu,
                    float* d_wd, int accumulate, char* ws, hipStream_t st) {
    return FINE_UNSUPPORTED;
}

}  // namespace fine
