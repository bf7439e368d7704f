// Internal: the fused 7 x 7 stride-2 convolution + ReLU + 3 x 3 stride-2 max-pool
// kernel (stem_pool.hip).
#pragma once
#include "fupr.h"

namespace fupr {

// True if the kernel covers this convolution (7 x 7, stride 2, pad 3, at most 4
// input channels, 64 filters, 16-bit) followed by this pool (3, 2, 1) on tensors
// with these channel strides.
bool stem_pool_applies(const fupr_conv_shape& s, fupr_dtype dt, int N, int H, int W, int xcs,
                       int ycs, int pool_k, int pool_stride, int pool_pad);
fupr_status launch_stem_pool(const fupr_conv_shape& s, fupr_dtype dt, int N, int H, int W, int xcs,
                             int ycs, const void* x, const void* packed, void* y, void* stream);

}  // namespace fupr
