// Binary 3x3 convolution: host-side dispatch to the small-problem kernel (bconv_small.hip) or to
// the tile kernel set for the layer's channel width (bconv_kernel.h, instantiated by bconv_inst.hip).
#include <stdlib.h>

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
    // a handful of images: the latency kernel (one block per 32 pixels x 32 channels), unless the
    // environment asks for the tile kernels (BNN_CONV_TILES_ONLY=1: lets tests reach them with
    // small shapes)
    const char *tiles_only = getenv("BNN_CONV_TILES_ONLY");
    if (!(tiles_only && tiles_only[0] && tiles_only[0] != '0')) {
        const bnn_status small = launch_conv_binary_small(in, n, h, w, c_in, wt, c_out, ep, s);
        if (small != BNN_ERR_UNSUPPORTED) return small;
    }
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
