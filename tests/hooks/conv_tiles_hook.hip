// Test hook, built into tests/hooks/libbnn_test_hooks.so only (never into libbnn.so): runs
// bnn_conv_binary's argument checks and then the persistent tile kernels for ANY supported shape,
// so that parity tests can put small and ragged shapes on the kernels that the library itself
// reserves for large layers (it sends small layers to its latency kernel).  Links against
// libbnn.so and reaches two of its internal C++ functions.
#include "bnn_internal.h"

extern "C" bnn_status bnn_test_conv_binary_tiles(const uint32_t *in_dev, int n, int h, int w, int c_in,
                                                 const uint32_t *w_dev, int c_out, const bnn_epilogue *ep,
                                                 int32_t *preact_out_dev, uint32_t *packed_out_dev,
                                                 void *stream)
{
    bnn::EpiArgs ea;
    const bnn_status st =
        bnn::check_conv_binary(in_dev, n, h, w, c_in, w_dev, c_out, ep, preact_out_dev, packed_out_dev, &ea);
    if (st != BNN_OK) return st;
    return bnn::launch_conv_binary_tiles(in_dev, n, h, w, c_in, w_dev, c_out, ea, (hipStream_t)stream);
}

// Which kernel bnn_conv_binary (tiles_only == 0) or the hook above (tiles_only != 0) runs a shape
// on: 10 = small-problem kernel, 3 = 256 x 128 tile, 2 = 128 x 128 tile with streamed weights,
// 1 = 128 x 128, 0 = 64 x 64, -1 = unsupported.  Host-only.
extern "C" int bnn_test_conv_binary_kernel_choice(int n, int h, int w, int c_in, int c_out, int tiles_only)
{
    return bnn::conv_binary_kernel_choice(n, h, w, c_in, c_out, tiles_only != 0);
}
