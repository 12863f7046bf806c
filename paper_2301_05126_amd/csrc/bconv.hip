// Binary 3x3 convolution: host-side dispatch to the small-problem kernel (bconv_small.hip) or to
// the tile kernel set for the layer's channel width (bconv_kernel.h, instantiated by bconv_inst.hip).
#include "bnn_internal.h"

namespace bnn {

#define BNN_DECL_WPH(N)                                                                                   \
    bnn_status launch_conv_binary_wph##N(const uint32_t *in, int n, int h, int w, int c_in,               \
                                         const uint32_t *wt, int c_out, const EpiArgs &ep, hipStream_t s); \
    int conv_tile_choice_wph##N(int n, int h, int w, int c_in, int c_out);
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

static int words_per_half(int c_in)
{
    // words per lane half per tap: channel words per pixel rounded up to 2, 4, 8, 16 or 32
    const int cw = (c_in + 31) / 32;
    int wph = 1;
    while (2 * wph < cw) wph *= 2;
    return wph;
}

int conv_binary_kernel_choice(int n, int h, int w, int c_in, int c_out, bool tiles_only)
{
    if (!conv_binary_supported(h, w, c_in) || n <= 0 || c_out <= 0) return -1;
    if (!tiles_only && conv_binary_small_qualifies(n, h, w, c_in, c_out)) return 10;
    switch (words_per_half(c_in)) {
    case 1: return conv_tile_choice_wph1(n, h, w, c_in, c_out);
    case 2: return conv_tile_choice_wph2(n, h, w, c_in, c_out);
    case 4: return conv_tile_choice_wph4(n, h, w, c_in, c_out);
    case 8: return conv_tile_choice_wph8(n, h, w, c_in, c_out);
    case 16: return conv_tile_choice_wph16(n, h, w, c_in, c_out);
    }
    return -1;
}

bnn_status launch_conv_binary_tiles(const uint32_t *in, int n, int h, int w, int c_in, const uint32_t *wt,
                                    int c_out, const EpiArgs &ep, hipStream_t s)
{
    if (n == 0) return BNN_OK;
    switch (words_per_half(c_in)) {
    case 1: return launch_conv_binary_wph1(in, n, h, w, c_in, wt, c_out, ep, s);
    case 2: return launch_conv_binary_wph2(in, n, h, w, c_in, wt, c_out, ep, s);
    case 4: return launch_conv_binary_wph4(in, n, h, w, c_in, wt, c_out, ep, s);
    case 8: return launch_conv_binary_wph8(in, n, h, w, c_in, wt, c_out, ep, s);
    case 16: return launch_conv_binary_wph16(in, n, h, w, c_in, wt, c_out, ep, s);
    }
    return BNN_ERR_UNSUPPORTED;
}

bnn_status launch_conv_binary(const uint32_t *in, int n, int h, int w, int c_in, const uint32_t *wt,
                              int c_out, const EpiArgs &ep, hipStream_t s)
{
    if (n == 0) return BNN_OK;
    // a handful of images: the latency kernel (one block per 32 pixels x 32 channels); the choice
    // depends on the layer's shape only
    const bnn_status small = launch_conv_binary_small(in, n, h, w, c_in, wt, c_out, ep, s);
    if (small != BNN_ERR_UNSUPPORTED) return small;
    return launch_conv_binary_tiles(in, n, h, w, c_in, wt, c_out, ep, s);
}

}  // namespace bnn
