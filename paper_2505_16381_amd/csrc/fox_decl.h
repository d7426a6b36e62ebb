// Scan kernel of the PaTH-FoX extension.
#pragma once
#include "path_common.h"

namespace path {

struct ScanArgs {
    const void* in;      // [BH][in_stride], first n_in entries of a row are read (the rest count as zero)
    const float* minus;  // optional (float input only): subtracted from `in` element by element before the scan
    void* out;           // [BH][out_stride], first n_out entries of a row are written
    int in_stride, out_stride, n_in, n_out;
    int inclusive;
    float scale_out;
    // in_user / out_user != 0: that side is one of the caller's per-token scalar tensors, addressed through
    // `ul` (batch, head and token strides) instead of [BH][stride] with unit token stride
    int in_user, out_user;
    UserLayout ul;
};
hipError_t launch_fox_scan(const ScanArgs& a, int BH, int in_type, int out_type, hipStream_t st);   // types: 0 float, 1 bf16

}  // namespace path
