// Which convolution kernel serves a geometry, and the tiling facts the plan
// needs for FLOP accounting.  Host only.
#include "launch.h"

namespace {
struct Inst { int nt, khm, ksm, occ; };
#define FC_ROW(NT_, KHM_, KSM_, OCC_) {NT_, KHM_, KSM_, OCC_},
const Inst kInst[] = {FC_STREAM_INSTANCES(FC_ROW)};
#undef FC_ROW
const int kNumInst = (int)(sizeof(kInst) / sizeof(kInst[0]));

int max_ksteps(ConvGeom g, int band, int cols) {
    g.band = band;
    int worst = 0;
    for (int n0 = 0; n0 < g.NCo; n0 += cols) {
        int e_lo, e_hi;
        fc_band_window(g, n0, n0 + cols, g.epc, &e_lo, &e_hi);
        int k = (e_hi - e_lo + 2 * g.epc - 1) / (2 * g.epc);  // K-steps of two chunks
        if (k > worst) worst = k;
    }
    return worst;
}
}  // namespace

// Conditions shared by the vector kernels.
static bool vector_ok(const ConvGeom &g) {
    // Operand side: folded channels and the filter window in multiples of the operand chunk (8 elements of a
    // 16-bit type, or 4 where F*C_in allows no more; 4 or 2 of fp32).  Output side: columns and stored rows in
    // multiples of a 16-byte chunk.
    const int E = g.epc, EO = 16 / g.eb;
    if (!((g.eb == 2 && (E == 8 || E == 4)) || (g.eb == 4 && (E == 4 || E == 2)))) return false;
    if (g.FC % E != 0 || g.kwin % E != 0 || g.NCo % EO != 0 || g.out_row % EO != 0) return false;
    // 32-bit byte offsets into x and into the packed filter, 32-bit chunk index into y.
    const long long eb = g.eb;
    const long long x_elems = (long long)g.N * g.H * g.in_row;
    const long long y_elems = (long long)g.N * g.Hout * g.out_row;
    const long long w_elems = (long long)g.KH * g.kwin * g.NCo;
    if ((x_elems + 4LL * g.in_row) * eb >= (1LL << 31) || y_elems / EO >= (1LL << 32) || w_elems * eb >= (1LL << 31)) return false;
    return true;
}

// the LDS-tiled kernel and the two variants of the streaming kernel below exist for the 16-bit types in
// 16-byte operand chunks only
bool fc_tiled_ok(const ConvGeom &g) { return g.eb == 2 && g.epc == 8 && vector_ok(g); }

int fc_tiled_bn(const ConvGeom &g) {
    // Multiplies issued by a tile width = sum over its N tiles of (K blocks inside the tile's band
    // window, or all of them for the dense walk) x (tile width).  A wider tile covers more output
    // slots, hence a wider band window and more structural zeros multiplied, and it pads F*C_out
    // further; but it moves fewer operand bytes per multiply and needs fewer workgroups.  The
    // weights are the measured time per issued multiply relative to the 128-column tile.
    static const struct { int bn; double weight; } kCand[] = {{128, 1.0}, {192, 0.93}, {256, 0.85}};
    int best = 128;
    double best_cost = 0.0;
    for (const auto &c : kCand) {
        double work = 0.0;
        for (int n0 = 0; n0 < g.NCo; n0 += c.bn) {
            int e_lo, e_hi;
            fc_band_window(g, n0, n0 + c.bn, 8, &e_lo, &e_hi);
            work += (double)((e_hi - e_lo + 31) / 32) * c.bn;
        }
        const double cost = work * c.weight;
        if (best_cost == 0.0 || cost < best_cost) best = c.bn, best_cost = cost;
    }
    return best;
}

bool fc_stream_shape(const ConvGeom &g, int band, StreamShape *out) {
    if (!vector_ok(g)) return false;
    // exact multiply-high division of (tile start + lane) by the folded width and by the output height
    if (g.Wf_out >= 65000 || g.Hout >= 65000) return false;
    // 32-bit byte offsets from a tile's first output row to its last (up to 33 rows further on)
    if (34LL * g.out_row * g.eb >= (1LL << 31) || 34LL * g.NCo * g.eb >= (1LL << 31)) return false;
    // 64 columns per wave first: for the small-C_in layers this is one K-step per kh with the
    // fewest structural-zero products; wider waves only when no such instance fits.
    static const int prefer[] = {2, 4};
    for (int nt : prefer) {
        if (g.eb == 4 && nt > 2) continue;  // fp32: 64 columns per wave only (LDS for the waves' output slabs)
        const int ks = max_ksteps(g, band, 32 * nt);
        // Beyond a dozen K-steps per tile the layer is bound by the matrix cores, not by the
        // output stream, and the LDS-tiled kernel (operands shared by four waves) is the better
        // tool.  The dense walk of a small-K layer may still use the largest instance.
        // (Where the tiled kernel does not serve the layer (fp32, 8-byte operand chunks) any instance that
        // fits is better than the element-gather kernel.)
        if (band && fc_tiled_ok(g) && g.KH * ks > 12) continue;
        for (int i = 0; i < kNumInst; ++i)
            if (kInst[i].nt == nt && g.KH <= kInst[i].khm && ks <= kInst[i].ksm) {
                out->inst = i;
                out->nt = nt;
                out->ksteps = ks;
                return true;
            }
    }
    return false;
}

bool fc_stream_lds_ok(const ConvGeom &g) {
    if (g.eb != 2 || g.epc != 8 || !vector_ok(g)) return false;
    if (g.Wf_out >= 65000 || g.Hout >= 65000) return false;
    if (34LL * g.out_row * 2 >= (1LL << 31) || 34LL * g.NCo * 2 >= (1LL << 31)) return false;
    if (g.M >= (1LL << 31) - (1LL << 20)) return false;
    // four waves of 64 columns per workgroup; compiled instance: KH = 3 and 18 chunks of 8 K values per kh
    // (F*C_in = 48 with KW' = 3: the first-layer shapes)
    if (g.NCo % 256 != 0 || g.NCo / 256 > 32) return false;
    // stored rows are whole folded rows (kept folded, or the reconstruct is an alias)
    if (g.out_row != g.Wf_out * g.NCo) return false;
    return g.KH == 3 && g.kwin == 18 * 8;
}

bool fc_stream_nchw_ok(const ConvGeom &g, int band, bool height_fold, int *ksteps) {
    // g.out_row is the plan's unfolded W_out here: elements per channel row of y for a width fold, rows per
    // channel plane for a height fold (the plan is the transposed image's).
    // one wave per 64 columns, at most 16 waves, 4 channels per LDS read
    if (g.eb != 2 || g.epc != 8 || g.FC % 8 != 0 || g.kwin % 8 != 0 || g.Co % 4 != 0) return false;
    if (g.NCo % 64 != 0 || g.NCo > 1024) return false;
    if (height_fold) {
        // 16-byte pieces run along the image width = the plan's rows: whole pieces of 8 columns; a thread of the
        // write-out serves the slots hg and hg + F/2
        if (g.Hout % 8 != 0 || g.F % 2 != 0 || g.out_row > g.F * g.Wf_out) return false;
    } else {
        // whole 16-byte pieces of 8 slots; every slot of every folded output pixel is a real output column
        if (g.F % 8 != 0 || g.out_row != g.F * g.Wf_out) return false;
    }
    if (g.Wf_out >= 65000 || g.Hout >= 65000) return false;
    // 32-bit byte offsets into x, y and the packed filter; 32-bit pixel and tile indices
    const long long x_elems = (long long)g.N * g.H * g.in_row;
    const long long y_elems = (long long)g.N * g.Co * g.Hout * g.out_row;
    const long long w_elems = (long long)g.KH * g.kwin * g.NCo;
    if (x_elems + 4LL * g.in_row >= (1LL << 30) || y_elems >= (1LL << 31) - 64 || w_elems >= (1LL << 30)) return false;
    if (g.M >= (1LL << 31) - (1LL << 20)) return false;
    const int ks = max_ksteps(g, band, 64);
    // compiled instances: (KH <= 1, two K-steps per kh) and (KH <= 3, one K-step per kh)
    if (!((g.KH <= 1 && ks <= 2) || (g.KH <= 3 && ks <= 1))) return false;
    *ksteps = ks;
    return true;
}

bool fc_stream_nchw_stage(const ConvGeom &g, NchwStage *out) {
    const long long W = (long long)g.Wf * g.F;
    // 16-byte pieces of 8 image columns; no tile crosses an image; the folded output is no wider than the input
    if (g.eb != 2 || W % 8 != 0 || ((long long)g.Hout * g.Wf_out) % 32 != 0 || g.Wf_out > g.Wf) return false;
    if (g.e_min > 0 || g.e_max < g.FC) return false;
    // output rows a tile of 32 consecutive folded pixels can touch, and the input rows under them
    const int rows = (g.Wf_out - 1 + 31) / g.Wf_out + 1 + g.KH - 1;
    const long long halo_l = -(long long)g.e_min, halo_r = (long long)g.e_max - g.FC;
    const long long pitch = ((halo_l + g.in_row + halo_r) * 2 + 15) / 16 * 16;
    if (halo_l % 8 != 0 || (long long)rows * g.C * (W / 8) > g.NCo) return false;  // one piece per thread and tile
    const long long lds = 2LL * 32 * (g.NCo * 2 + 8) + 2LL * rows * pitch;
    if (lds > 163840) return false;
    out->rows = rows;
    out->pitch = (int)pitch;
    out->halo_l = (int)halo_l;
    out->lds_bytes = lds;
    return true;
}

int fc_choose_kernel(const ConvGeom &g, foldconv_dtype_t dt) {
    // Channel counts that miss the chunk alignment, and fp32 or 8-byte-chunk layers too large for the
    // streaming kernel's registers, run the element-gather MFMA kernel (the analogue of
    // Algorithm 1's fallback: it is correct for every shape, just not fast).
    (void)dt;  // element size and operand chunk are in g
    StreamShape sh;
    if (fc_stream_shape(g, 1, &sh)) return FC_KERNEL_STREAM;
    if (fc_tiled_ok(g)) return FC_KERNEL_TILED;
    return FC_KERNEL_GATHER;
}

int fc_band_tile_n(int kernel, const ConvGeom &g) {
    StreamShape sh;
    switch (kernel) {
        case FC_KERNEL_STREAM: return fc_stream_shape(g, 1, &sh) ? 32 * sh.nt : 32;
        case FC_KERNEL_TILED: return fc_tiled_bn(g);
        default: return 32;
    }
}

int fc_band_align(int kernel, const ConvGeom &g) {
    if (kernel == FC_KERNEL_GATHER) return 1;
    return g.epc;
}
