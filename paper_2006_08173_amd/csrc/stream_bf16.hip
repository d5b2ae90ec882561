// The streaming kernels for bf16 tensors (see stream_kernels.hpp).
#include "stream_kernels.hpp"

namespace lgn {

StreamKernel pick_stream_kernel_bf16(bool prune, bool quant, int rounding, int out_kind)
{
    return pick_kernel<LGN_BF16>(prune, quant, rounding, out_kind);
}

StreamBatchKernel pick_stream_batch_kernel_bf16(int rounding, int out_kind)
{
    return pick_batch_kernel<LGN_BF16>(rounding, out_kind);
}

}  // namespace lgn
