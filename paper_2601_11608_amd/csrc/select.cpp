// Which convolution kernel serves a geometry, and the tiling facts the plan
// needs for FLOP accounting.  Host only.
#include "launch.h"

int fc_choose_kernel(const ConvGeom &g, foldconv_dtype_t dt) {
    // fp32 and channel counts that miss the 16-byte chunk alignment run the
    // element-gather MFMA kernel (the analogue of Algorithm 1's fallback: it is
    // correct for every shape, just not fast).
    if (dt == FOLDCONV_F32) return FC_KERNEL_GATHER;
    if (g.FC % 8 != 0) return FC_KERNEL_GATHER;
    return FC_KERNEL_GATHER;
}

bool fc_stream_shape(const ConvGeom &, int, StreamShape *) { return false; }

int fc_band_tile_n(int kernel, const ConvGeom &) {
    switch (kernel) {
        case FC_KERNEL_TILED: return 128;
        default: return 32;
    }
}

int fc_band_align(int kernel, foldconv_dtype_t dt) {
    if (kernel == FC_KERNEL_GATHER) return 1;
    return dt == FOLDCONV_F32 ? 1 : 8;
}
