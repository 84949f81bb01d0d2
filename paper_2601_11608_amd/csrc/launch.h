// Internal interface between the host-side plan/ABI code and the HIP
// translation units.  Streams travel as void* so that plan.cpp stays free of
// HIP headers.
#pragma once
#include "geom.h"

// --- kernel choice and its tiling facts (select.cpp) -------------------------
int fc_choose_kernel(const ConvGeom &g, foldconv_dtype_t dt);
int fc_band_tile_n(int kernel, const ConvGeom &g);  // output columns sharing one band window
int fc_band_align(int kernel, foldconv_dtype_t dt); // alignment of the band window in elements

// Shape of the streaming kernel instance for a geometry; false if none fits.
struct StreamShape {
    int nt;      // 32-column MFMA tiles held per wave
    int ksteps;  // 16-wide K-steps per kh held per wave
};
bool fc_stream_shape(const ConvGeom &g, int band, StreamShape *out);

// --- launchers (return 0 or a hipError_t value) -------------------------------
int fc_launch_expand(const foldconv_plan_s *p, const void *w, void *w_exp, void *stream);
int fc_launch_copy(const void *src, void *dst, size_t bytes, void *stream);
int fc_launch_unfold(const foldconv_plan_s *p, const void *y_fold, void *y, void *stream);
int fc_launch_pad_input(const foldconv_plan_s *p, const void *x, void *x_pad, void *stream);
int fc_launch_pad_filter(const foldconv_plan_s *p, const void *w, void *w_pad, void *stream);
int fc_launch_pack(const ConvGeom &g, int elem_bytes, const void *w_exp, void *w_pack, void *stream);
int fc_launch_conv(int kernel, foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_exp,
                   const void *w_pack, const void *bias, void *y, void *stream);

// Per-kernel launchers behind fc_launch_conv.
int fc_launch_conv_gather(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_exp, const void *bias,
                          void *y, void *stream);
