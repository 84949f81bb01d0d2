// Routes a convolution to the kernel the plan chose.
#include "launch.h"

int fc_launch_conv(int kernel, foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_exp,
                   const void *w_pack, const void *bias, void *y, void *stream) {
    (void)w_pack;
    switch (kernel) {
        case FC_KERNEL_GATHER:
        default:
            return fc_launch_conv_gather(dt, g, x, w_exp, bias, y, stream);
    }
}
