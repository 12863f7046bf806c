// Binary 3x3 convolution: host-side dispatch to the kernel set for the layer's channel width.
// The kernels live in bconv_kernel.h and are instantiated by bconv_inst.hip.
#include "bnn_internal.h"

namespace bnn {

#define BNN_DECL_WPH(N)                                                                                   \
    bnn_status launch_conv_binary_wph##N(const uint32_t *in, int n, int h, int w, int c_in,               \
                                         const uint32_t *wt, int c_out, const EpiArgs &ep, hipStream_t s);
BNN_DECL_WPH(1)
BNN_DECL_WPH(2)
BNN_DECL_WPH(4)
BNN_DECL_WPH(8)
BNN_DECL_WPH(16)
#undef BNN_DECL_WPH

bool conv_binary_supported(int h, int w, int c_in)
{
    // at most 32 words per pixel (the smallest block tile then fits LDS); one image's packed
    // input below 2 GiB (32-bit byte offsets inside a block's buffer resource)
    return c_in <= 1024 && (int64_t)h * w * ((c_in + 31) / 32) * 4 < 0x7fffffffLL;
}

bnn_status launch_conv_binary(const uint32_t *in, int n, int h, int w, int c_in, const uint32_t *wt,
                              int c_out, const EpiArgs &ep, hipStream_t s)
{
    if (n == 0) return BNN_OK;
    // words per lane half per tap: channel words per pixel rounded up to 2, 4, 8, 16 or 32
    const int cw = (c_in + 31) / 32;
    int wph = 1;
    while (2 * wph < cw) wph *= 2;
    switch (wph) {
    case 1: return launch_conv_binary_wph1(in, n, h, w, c_in, wt, c_out, ep, s);
    case 2: return launch_conv_binary_wph2(in, n, h, w, c_in, wt, c_out, ep, s);
    case 4: return launch_conv_binary_wph4(in, n, h, w, c_in, wt, c_out, ep, s);
    case 8: return launch_conv_binary_wph8(in, n, h, w, c_in, wt, c_out, ep, s);
    case 16: return launch_conv_binary_wph16(in, n, h, w, c_in, wt, c_out, ep, s);
    }
    return BNN_ERR_UNSUPPORTED;
}

}  // namespace bnn
