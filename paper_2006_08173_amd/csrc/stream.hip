// Launch side of the streaming operators (kernels: stream_kernels.hpp) and the dequantizer.
#include "stream_kernels.hpp"

namespace lgn {

// ---- dequantize (not on the hot path): one element per thread ------------------------------
template <int DTYPE, int IN_KIND>
__global__ __launch_bounds__(kBlock) void dequant_kernel(const uint8_t *__restrict__ codes,
                                                         uint64_t n, const lgn_fp_params_t *f,
                                                         void *out)
{
    QuantConst q;
    load_quant_const(f, q);
    const uint64_t total_bytes = (n * (uint64_t)q.n_bits + 7) / 8;
    const uint64_t gsize = (uint64_t)gridDim.x * kBlock;
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += gsize) {
        uint32_t code;
        if (IN_KIND == LGN_OUT_CODE8) {
            code = codes[i];
        } else {
            const uint64_t bit = i * (uint64_t)q.n_bits, byte = bit >> 3;
            uint32_t win = codes[byte];
            if (byte + 1 < total_bytes) win |= (uint32_t)codes[byte + 1] << 8;
            code = (win >> (bit & 7)) & ((1u << q.n_bits) - 1u);
        }
        store_elem<DTYPE>(out, i, code_value_bits(code, q));
    }
}

// Workgroups of one tensor's streaming grid.  A wave gets a few pairs of tiles, so that there are
// far more workgroups than the device holds at once: they start staggered, and the waves' load
// and arithmetic phases do not march in step (fp32, fused pass of 205 M elements: 8 workgroups per
// CU with ~50 pairs per wave 0.200 ms, ~65 per CU with 6 pairs 0.180 ms).  The passes over fp32
// tensors are bound by memory and like 3 to 6 pairs (fused pass after a statistics pass: 282.6 /
// 283.7 / 284.5 / 288 / 291 / 298 us per step at 3 / 4 / 6 / 8 / 12 / 16).  The 16-bit types carry
// twice the elements per byte and are bound by instruction issue; there the per-wave set-up
// weighs more than the staggering (10^9 bf16 elements to packed 6-bit codes: 752 / 687 / 669 / 660 /
// 655 / 651 / 651 / 653 us at 3 / 6 / 8 / 12 / 16 / 24 / 32 / 48).
static uint64_t stream_grid(uint64_t n, int dtype)
{
    const uint64_t npairs = ((n + 255) / 256 + 1) / 2;
    const long knob = tuning(LGN_TUNE_STREAM_PAIRS_PER_WAVE);
    const uint64_t per_wave = knob > 0 ? (uint64_t)knob : (dtype == LGN_F32 ? 6 : 24);
    const uint64_t per_block = per_wave * (kBlock / kWave);
    uint64_t blocks = (npairs + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    const uint64_t max_blocks = (uint64_t)device_cus() * (uint64_t)tuning(LGN_TUNE_STREAM_BLOCKS_PER_CU);
    return blocks > max_blocks ? max_blocks : blocks;
}

hipError_t launch_stream(int dtype, bool prune, bool quant, int rounding, int out_kind,
                         const StreamArgs &args, hipStream_t stream)
{
    if (args.n == 0) return hipSuccess;
    StreamKernel k;
    if (dtype == LGN_F32) k = pick_stream_kernel_f32(prune, quant, rounding, out_kind);
    else if (dtype == LGN_BF16) k = pick_stream_kernel_bf16(prune, quant, rounding, out_kind);
    else k = pick_stream_kernel_f16(prune, quant, rounding, out_kind);
    const uint64_t blocks = stream_grid(args.n, dtype);
    hipLaunchKernelGGL(k, dim3((unsigned)blocks), dim3(kBlock), 0, stream, args);
    return hipGetLastError();
}

// The fused pass over `count` tensors, kBatchMax tensors per launch.  Empty tensors get no
// workgroups.
hipError_t launch_batch_stream(const lgn_batch_item_t *items, int count, int dtype, int rounding,
                               int out_kind, hipStream_t stream)
{
    StreamBatchKernel k;
    if (dtype == LGN_F32) k = pick_stream_batch_kernel_f32(rounding, out_kind);
    else if (dtype == LGN_BF16) k = pick_stream_batch_kernel_bf16(rounding, out_kind);
    else k = pick_stream_batch_kernel_f16(rounding, out_kind);
    int i = 0;
    while (i < count) {
        BatchStreamArgs a;
        uint64_t next = 0;
        int m = 0;
        for (int j = 0; j < kBatchMax; ++j) {
            a.first_block[j] = 0xffffffffu;
            a.t[j] = BatchStreamTensor{};
        }
        // fill the table with the next non-empty tensors, as long as the grid index fits 31 bits
        while (i < count && m < kBatchMax) {
            const lgn_batch_item_t &it = items[i];
            if (it.n == 0) { ++i; continue; }
            const uint64_t blocks = stream_grid(it.n, dtype);
            if (m > 0 && next + blocks > 0x7fffffffull) break;
            BatchStreamTensor &T = a.t[m];
            T.g = it.g; T.out = it.out; T.n = it.n; T.p = it.p; T.f = it.f;
            T.k0 = (uint32_t)it.seed; T.k1 = (uint32_t)(it.seed >> 32);
            T.blocks = (uint32_t)blocks;
            a.first_block[m] = (uint32_t)next;
            next += blocks;
            ++m; ++i;
        }
        if (m == 0) break;
        hipLaunchKernelGGL(k, dim3((unsigned)next), dim3(kBlock), 0, stream, a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_dequant(const void *codes, uint64_t n, int in_kind, const lgn_fp_params_t *f,
                          int dtype, void *out, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    uint64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 65536) blocks = 65536;
    const uint8_t *c = static_cast<const uint8_t *>(codes);
    if (dtype == LGN_F32) {
        if (in_kind == LGN_OUT_CODE8) dequant_kernel<LGN_F32, LGN_OUT_CODE8><<<blocks, kBlock, 0, stream>>>(c, n, f, out);
        else dequant_kernel<LGN_F32, LGN_OUT_PACKED><<<blocks, kBlock, 0, stream>>>(c, n, f, out);
    } else if (dtype == LGN_BF16) {
        if (in_kind == LGN_OUT_CODE8) dequant_kernel<LGN_BF16, LGN_OUT_CODE8><<<blocks, kBlock, 0, stream>>>(c, n, f, out);
        else dequant_kernel<LGN_BF16, LGN_OUT_PACKED><<<blocks, kBlock, 0, stream>>>(c, n, f, out);
    } else {
        if (in_kind == LGN_OUT_CODE8) dequant_kernel<LGN_F16, LGN_OUT_CODE8><<<blocks, kBlock, 0, stream>>>(c, n, f, out);
        else dequant_kernel<LGN_F16, LGN_OUT_PACKED><<<blocks, kBlock, 0, stream>>>(c, n, f, out);
    }
    return hipGetLastError();
}

}  // namespace lgn
