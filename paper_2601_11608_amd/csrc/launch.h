// Internal interface between the host-side plan/ABI code and the HIP
// translation units.  Streams travel as void* so that plan.cpp stays free of
// HIP headers.
#pragma once
#include "geom.h"

// --- kernel choice and its tiling facts (select.cpp) -------------------------
int fc_choose_kernel(const ConvGeom &g, foldconv_dtype_t dt);
int fc_band_tile_n(int kernel, const ConvGeom &g);  // output columns sharing one band window (for g's walk, g.band)
int fc_band_align(int kernel, const ConvGeom &g);   // alignment of the band window in elements

// Shape of the streaming kernel instance for a geometry; false if none fits.
struct StreamShape {
    int inst;    // index into FC_STREAM_INSTANCES
    int nt;      // 32-column MFMA tiles held per wave
    int ksteps;  // K-steps (two operand chunks each) per kh actually walked
};
// Compiled instances of the streaming kernel: X(NT, max KH, max K-steps per kh, workgroups per CU).
// Filter fragments cost 4*NT*KH*ksteps registers per lane, which bounds the list.
#define FC_STREAM_INSTANCES(X) \
    X(2, 1, 1, 2) X(2, 3, 1, 2) X(2, 5, 1, 2) X(2, 1, 2, 2) X(2, 3, 2, 2) X(2, 3, 3, 2) X(2, 3, 4, 2) X(2, 1, 6, 2) X(2, 3, 9, 1) \
    X(4, 1, 2, 2) X(4, 3, 2, 2)
bool fc_stream_shape(const ConvGeom &g, int band, StreamShape *out);

// --- the GPU the calling thread is on (device_info.hip); returns 0 or a hipError_t value ----------
struct FcDevice {
    unsigned cus;   // compute units
    unsigned xcds;  // accelerator dies, each with its own L2; workgroup b is placed on die b % xcds
    unsigned wall_khz;  // rate of the constant clock wall_clock64() reads in a kernel, 0 = unknown
};
int fc_device(FcDevice *out);

// --- store pacing of the persistent streaming kernels ---------------------------------------------
// A write-dominated launch whose waves offer the memory system more than it can take runs 10-20 %
// below what the same store stream reaches when every wave issues its bursts on a fixed schedule just
// under that rate (a stand-alone stream of this kernel's store pattern, 411 MB: 69-72 us unpaced,
// 59 us paced at 7.4 TB/s offered, 64 us at 7.8, 62 us for a plain fill).  The kernels therefore hold
// each wave's store burst back until its slot on the constant wall clock.  Returns the interval between
// a wave's bursts in wall-clock ticks * 256 when the launch moves `bytes` (input read once + output) in
// `tiles_per_wave` equal steps at kPaceBytesPerSecond, or 0 (unpaced) for launches too short to reach
// that steady state and where the clock rate is unknown.
constexpr double kPaceBytesPerSecond = 7.35e12;
inline unsigned fc_store_pace(double bytes, unsigned tiles_per_wave, unsigned wall_khz,
                              double bytes_per_second = kPaceBytesPerSecond) {
    if (wall_khz == 0 || tiles_per_wave < 12 || bytes < 64e6) return 0;
    const double ticks = bytes / bytes_per_second / tiles_per_wave * (double)wall_khz * 1e3;
    return ticks * 256.0 < 4e9 ? (unsigned)(ticks * 256.0) : 0u;
}

// --- foldconv_forward's body (api.cpp).  remember_workspace = false: the packed filter goes to a
//     buffer the caller of the ABI never sees, so the plan does not record it as a prepared workspace.
int fc_forward(foldconv_plan_t plan, const void *x_fold, const void *w_exp, const void *bias, void *y, void *workspace,
               size_t workspace_bytes, unsigned flags, void *stream, bool remember_workspace);

// --- launchers (return 0 or a hipError_t value) -------------------------------
int fc_launch_expand(const foldconv_plan_s *p, const void *w, void *w_exp, int oihw, void *stream);
int fc_launch_fold_nchw(const foldconv_plan_s *p, const void *x, void *x_fold, void *stream);
int fc_launch_unfold_nchw(const foldconv_plan_s *p, const void *y_fold, void *y, void *stream);
int fc_launch_copy(const void *src, void *dst, size_t bytes, void *stream);
int fc_launch_unfold(const foldconv_plan_s *p, const void *y_fold, void *y, void *stream);
int fc_launch_pad_input(const foldconv_plan_s *p, const void *x, void *x_pad, void *stream);
int fc_launch_pad_filter(const foldconv_plan_s *p, const void *w, void *w_pad, void *stream);
int fc_launch_pad_bias(const foldconv_plan_s *p, const void *b, void *b_pad, void *stream);
int fc_launch_crop_channels(const foldconv_plan_s *p, const void *y_pad, void *y, void *stream);
int fc_launch_pack(const ConvGeom &g, int elem_bytes, const void *w_exp, void *w_pack, void *stream);
int fc_launch_compact(const ConvGeom &g, int elem_bytes, const void *w, void *w_compact, void *stream);
int fc_launch_conv(int kernel, foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_exp,
                   const void *w_pack, const void *bias, void *y, void *stream);

// Per-kernel launchers behind fc_launch_conv.
int fc_launch_conv_stream(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_pack, const void *bias,
                          void *y, void *stream);
int fc_launch_conv_tiled(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_pack, const void *bias,
                         void *y, void *stream);
// Streaming kernel that writes a channels-first output (g.out_row = the plan's unfolded W_out: the image's
// W_out for a width fold, its H_out for a height fold, whose plan is that of the transposed image); false
// if the geometry does not fit it.
bool fc_stream_nchw_ok(const ConvGeom &g, int band, bool height_fold, int *ksteps);
// Width folds that read a channels-first input stage its rows through LDS behind the two output tiles: rows per
// stage buffer, bytes per row (zero halo, the folded row, zero halo) and elements of the halo in front; false where
// that does not fit (an image must be a whole number of 32-pixel tiles, one 16-byte piece per thread and tile, 160 KB
// of LDS in all).
struct NchwStage { int rows, pitch, halo_l; long long lds_bytes; };
bool fc_stream_nchw_stage(const ConvGeom &g, NchwStage *out);
// x_nchw: x is the channels-first input itself (same bytes as x' otherwise): gathered element by element (height
// fold) or staged through LDS (width fold, where fc_stream_nchw_stage allows).
int fc_launch_conv_stream_nchw(foldconv_dtype_t dt, const ConvGeom &g, bool height_fold, bool x_nchw, const void *x,
                               const void *w_pack, const void *bias, void *y, void *stream);
// Streaming kernel with the input tile staged through LDS (dense walks whose K extent fits the registers).
bool fc_stream_lds_ok(const ConvGeom &g);
int fc_launch_conv_stream_lds(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_pack,
                              const void *bias, void *y, void *stream);
bool fc_tiled_ok(const ConvGeom &g);
int fc_tiled_bn(const ConvGeom &g);  // output columns per workgroup tile of the tiled kernel for g's walk (g.band): 128, 192 or 256
int fc_launch_conv_gather(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_exp, const void *bias,
                          void *y, void *stream);
