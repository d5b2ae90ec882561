// The streaming kernels for f32 tensors (see stream_kernels.hpp).
#include "stream_kernels.hpp"

namespace lgn {

StreamKernel pick_stream_kernel_f32(bool prune, bool quant, int rounding, int out_kind)
{
    return pick_kernel<LGN_F32>(prune, quant, rounding, out_kind);
}

StreamBatchKernel pick_stream_batch_kernel_f32(int rounding, int out_kind)
{
    return pick_batch_kernel<LGN_F32>(rounding, out_kind);
}

}  // namespace lgn
