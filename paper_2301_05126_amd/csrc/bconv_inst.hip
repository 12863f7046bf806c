// One instantiation set of the binary 3x3 convolution kernels for one channel-word width,
// compiled once per BNN_CONV_WPH and BNN_CONV_PART so the sets build in parallel:
// part 0 = dispatcher and the smaller block tiles, part 1 = the 256 x 128 tile.
#include "bconv_kernel.h"

#if !defined(BNN_CONV_WPH) || !defined(BNN_CONV_PART)
#error "compile with -DBNN_CONV_WPH={1,2,4,8,16} -DBNN_CONV_PART={0,1}"
#endif

#define BNN_CAT2(a, b) a##b
#define BNN_CAT(a, b) BNN_CAT2(a, b)

namespace bnn {

#if BNN_CONV_PART == 0
bnn_status BNN_CAT(launch_conv_binary_wph, BNN_CONV_WPH)(const uint32_t *in, int n, int h, int w, int c_in,
                                                         const uint32_t *wt, int c_out, const EpiArgs &ep,
                                                         hipStream_t s)
{
    return launch_wph<BNN_CONV_WPH>(in, wt, n, h, w, c_in, c_out, ep, s);
}

int BNN_CAT(conv_tile_choice_wph, BNN_CONV_WPH)(int n, int h, int w, int c_in, int c_out)
{
    return tile_choice_wph<BNN_CONV_WPH>(n, h, w, c_in, c_out);
}
#else
template <>
bnn_status launch_conv_big_tile<BNN_CONV_WPH>(const uint32_t *in, const uint32_t *wt, int n, int h, int w,
                                              int c_in, int c_out, const EpiArgs &ep, hipStream_t s)
{
    return launch_one<4, 2, BNN_CONV_WPH, (BNN_CONV_WPH >= 8)>(in, wt, n, h, w, c_in, c_out, ep, s);
}
#endif

}  // namespace bnn
