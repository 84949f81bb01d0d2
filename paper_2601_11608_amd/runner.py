"""Per-layer and per-stack call sequences over the C ABI (buffer ownership and
call order only; all computation happens inside libfoldconv's kernels)."""
import torch

from . import binding as fc


class FoldedLayer:
    """One convolution layer prepared once (plan, expanded + packed filter) and
    then run many times, as the paper's post-training rewrite intends."""

    def __init__(self, layer, w, b, device="cuda"):
        self.layer = layer
        self.dtype = w.dtype
        self.plan = fc.foldconv_plan(*layer.plan_args(), w.dtype)
        s = self.plan.shapes
        self.w = w.to(device).contiguous()
        self.b = None if b is None else b.to(device).contiguous()
        self.w_exp = torch.empty(s.w_exp_bytes // s.elem_bytes, dtype=w.dtype, device=device)
        fc.foldconv_expand_filter(self.plan, self.w, self.w_exp)
        self.ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device=device)
        fc.foldconv_pack_filter(self.plan, self.w_exp, self.ws)
        self.ws_pad = None
        self.pad_ready = False
        self.ws_compact = None

    def out_shape(self):
        s = self.plan.shapes
        return (s.N, s.H_out, s.W_out, s.C_out)

    def new_output(self):
        return torch.empty(self.out_shape(), dtype=self.dtype, device=self.w.device)

    def forward(self, x, y, flags=0, repack=False, compact=False):
        """fold (aliased: x' shares x's bytes) + folded convolution + fused reconstruct.
        compact=True runs from the compact filter (non-zero blocks only), built once from w;
        compact=None takes the plan's hint (shapes.prefer_compact)."""
        if compact is None:
            compact = bool(self.plan.shapes.prefer_compact)
        fc.foldconv_fold_input(self.plan, x, x)
        if self.layer.relu:
            flags |= fc.FLAG_RELU
        if compact:
            if self.ws_compact is None:
                n = max(int(self.plan.shapes.filter_compact_bytes), 256)
                self.ws_compact = torch.empty(n, dtype=torch.uint8, device=self.w.device)
                fc.foldconv_pack_filter_compact(self.plan, self.w, self.ws_compact)
            fc.foldconv_forward(self.plan, x, None, self.b, y, self.ws_compact, flags | fc.FLAG_FILTER_COMPACT)
            return y
        if not repack:
            flags |= fc.FLAG_FILTER_PACKED
        fc.foldconv_forward(self.plan, x, self.w_exp, self.b, y, self.ws, flags)
        return y

    def forward_padded(self, x, y, repack=False):
        s = self.plan.shapes
        if self.ws_pad is None:
            self.ws_pad = torch.empty(max(int(s.padded_workspace_bytes), 256), dtype=torch.uint8, device=self.w.device)
        flags = fc.FLAG_RELU if self.layer.relu else 0
        if self.pad_ready and not repack:
            flags |= fc.FLAG_FILTER_PACKED
        fc.conv_padded_forward(self.plan, x, self.w, self.b, y, self.ws_pad, flags)
        self.pad_ready = True
        return y


class FoldedStack:
    """A chain of layers; each output buffer is the next layer's (aliased) folded input."""

    def __init__(self, layers, ws, bs, device="cuda"):
        self.layers = [FoldedLayer(l, w, b, device) for l, w, b in zip(layers, ws, bs)]
        self.outs = [l.new_output() for l in self.layers]

    def forward(self, x, flags=0, padded=False, compact=False):
        """compact: False = packed w' everywhere, True = compact filter everywhere, None = per layer as the plan hints."""
        a = x
        for l, y in zip(self.layers, self.outs):
            if padded:
                l.forward_padded(a, y)
            else:
                l.forward(a, y, flags, compact=compact)
            a = y
        return a


class ChannelsFirstLayer:
    """One convolution layer on channels-first tensors: x [N][C_in][H][W], w [C_out][C_in][KH][KW],
    y [N][C_out][H_out][W_out].  The fold is a re-indexing kernel here; the convolution writes y
    channels-first itself where the plan allows it (shapes.out_nchw_fused), otherwise it writes the
    folded output and the reconstruct kernel re-indexes that."""

    def __init__(self, layer, w_oihw, b, fold_axis=fc.FOLD_W, device="cuda"):
        self.layer = layer
        self.dtype = w_oihw.dtype
        self.plan = fc.foldconv_plan_nchw(layer.N, layer.C_in, layer.H, layer.W, layer.C_out, layer.KH, layer.KW,
                                          layer.pad, layer.F, fold_axis, w_oihw.dtype)
        s = self.plan.shapes
        self.fused = bool(s.out_nchw_fused)
        self.one_launch = self.fused  # until a call says the geometry does not allow reading x channels-first
        self.w = w_oihw.to(device).contiguous()
        self.b = None if b is None else b.to(device).contiguous()
        self.w_exp = torch.empty(s.w_exp_bytes // s.elem_bytes, dtype=self.dtype, device=device)
        fc.foldconv_expand_filter_oihw(self.plan, self.w, self.w_exp)
        self.ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device=device)
        fc.foldconv_pack_filter(self.plan, self.w_exp, self.ws)
        self.x_fold = torch.empty(s.x_bytes // s.elem_bytes, dtype=self.dtype, device=device)
        self.y_fold = None if self.fused else torch.empty(s.y_fold_bytes // s.elem_bytes, dtype=self.dtype, device=device)

    def out_shape(self):
        s = self.plan.shapes
        if s.fold_axis == fc.FOLD_H:  # the plan describes the transposed image
            return (s.N, s.C_out, s.W_out, s.H_out)
        return (s.N, s.C_out, s.H_out, s.W_out)

    def new_output(self):
        return torch.empty(self.out_shape(), dtype=self.dtype, device=self.w.device)

    def forward(self, x, y):
        flags = fc.FLAG_FILTER_PACKED | (fc.FLAG_RELU if self.layer.relu else 0)
        if self.fused and self.one_launch:
            # one launch: the kernel reads x and writes y channels-first
            try:
                fc.foldconv_forward(self.plan, x, self.w_exp, self.b, y, self.ws, flags | fc.FLAG_OUT_NCHW | fc.FLAG_IN_NCHW)
                return y
            except fc.FoldconvError as e:
                if e.status != -3:  # unsupported: a width fold whose input rows do not fit LDS; fold first from now on
                    raise
                self.one_launch = False
        fc.foldconv_fold_input_nchw(self.plan, x, self.x_fold)
        if self.fused:
            fc.foldconv_forward(self.plan, self.x_fold, self.w_exp, self.b, y, self.ws, flags | fc.FLAG_OUT_NCHW)
        else:
            fc.foldconv_forward(self.plan, self.x_fold, self.w_exp, self.b, self.y_fold, self.ws,
                                flags | fc.FLAG_KEEP_FOLDED)
            fc.foldconv_unfold_output_nchw(self.plan, self.y_fold, y)
        return y
