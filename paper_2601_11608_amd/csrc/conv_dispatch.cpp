// Routes a convolution to the kernel the plan chose.
#include "launch.h"

int fc_launch_conv(int kernel, foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_exp,
                   const void *w_pack, const void *bias, void *y, void *stream) {
    switch (kernel) {
        case FC_KERNEL_STREAM: {
            // The dense walk may need more K-steps than any streaming instance holds;
            // the tiled kernel reads the same packed filter.
            StreamShape sh;
            // Dense walk with the whole K extent in registers: the variant that shares each input
            // tile among four waves through LDS.
            if (!g.band && fc_stream_lds_ok(g)) return fc_launch_conv_stream_lds(dt, g, x, w_pack, bias, y, stream);
            if (fc_stream_shape(g, g.band, &sh)) return fc_launch_conv_stream(dt, g, x, w_pack, bias, y, stream);
            // fp32 and 8-byte operand chunks have no tiled kernel; the element-gather kernel reads the canonical filter
            if (!fc_tiled_ok(g)) return fc_launch_conv_gather(dt, g, x, w_exp, bias, y, stream);
            return fc_launch_conv_tiled(dt, g, x, w_pack, bias, y, stream);
        }
        case FC_KERNEL_TILED:
            return fc_launch_conv_tiled(dt, g, x, w_pack, bias, y, stream);
        case FC_KERNEL_GATHER:
        default:
            return fc_launch_conv_gather(dt, g, x, w_exp, bias, y, stream);
    }
}
