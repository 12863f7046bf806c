// One instantiation set of the binary 3x3 convolution kernels (all block tiles for one
// channel-word width).  Compiled once per BNN_CONV_WPH so the sets build in parallel.
#include "bconv_kernel.h"

#ifndef BNN_CONV_WPH
#error "compile with -DBNN_CONV_WPH={1,2,4,8,16}"
#endif

#define BNN_CAT2(a, b) a##b
#define BNN_CAT(a, b) BNN_CAT2(a, b)

namespace bnn {

bnn_status BNN_CAT(launch_conv_binary_wph, BNN_CONV_WPH)(const uint32_t *in, int n, int h, int w, int c_in,
                                                         const uint32_t *wt, int c_out, const EpiArgs &ep,
                                                         hipStream_t s)
{
    return launch_wph<BNN_CONV_WPH>(in, wt, n, h, w, c_in, c_out, ep, s);
}

}  // namespace bnn
