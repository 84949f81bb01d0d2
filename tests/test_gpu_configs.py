"""The five benchmark configurations at full size, in the launch configuration
the benchmark times (prepared filter, aliased fold, fused reconstruct),
against the fp64 oracle: every image of the single-layer configurations, a
quarter of the images of the stack (images are independent), relative L2 per
image and an element-wise bound per layer; the whole output is checked for
unwritten (NaN-filled) elements."""
import numpy as np
import pytest
import torch

from helpers import TOL, assert_elementwise, f64, rel_l2_per_image

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import paper_2601_11608_amd as fc
    from paper_2601_11608_amd import runner, workloads

    fc.load_library()
    assert torch.cuda.is_available()
    return fc, runner, workloads


_ORACLE_CACHE = {}


def oracle_chain(oracle, name, layers, x, ws, bs, images):
    """fp64 chain over the sampled images, once per configuration (the four walks share it)."""
    if name not in _ORACLE_CACHE:
        a = f64(x[images])
        for l, w, b in zip(layers, ws, bs):
            ph, pw = oracle.axis_pads(l.KH, l.KW, l.pad)
            a = oracle.conv_direct(a, f64(w), None if b is None else f64(b), ph, pw, l.relu)
        _ORACLE_CACHE.clear()                      # one configuration at a time: the outputs are large
        _ORACLE_CACHE[name] = a
    return _ORACLE_CACHE[name]


def check_layer_elementwise(oracle, l, a_in, w, b, got, what):
    """One layer on the input the GPU itself consumed (so that rounding between layers does not
    enter): every output element within the accumulation + one-rounding bound of the oracle."""
    ph, pw = oracle.axis_pads(l.KH, l.KW, l.pad)
    wf, bf = f64(w), None if b is None else f64(b)
    ref = oracle.conv_direct(a_in, wf, bf, ph, pw, l.relu)
    S = oracle.conv_direct(np.abs(a_in), np.abs(wf), None if bf is None else np.abs(bf), ph, pw, False)
    return assert_elementwise(got, ref, S, l.KH * l.KW * l.C_in, l.dtype, what)


# every image of the single-layer configurations; 8 of the 32 images of the stack
CASES = [("c1", None), ("c2", None), ("c3", None), ("c4", None), ("c5", [0, 3, 7, 12, 16, 21, 26, 31])]


@pytest.mark.parametrize("name,images", CASES)
@pytest.mark.parametrize("mode", ["band", "dense", "padded", "compact"])
def test_config_matches_oracle(env, oracle, name, images, mode):
    fc, runner, wl = env
    layers, x, ws, bs = wl.make_config(name)
    images = list(range(layers[0].N)) if images is None else images
    print("config", name, mode, "images", len(images), flush=True)
    stack = runner.FoldedStack(layers, ws, bs)
    for y in stack.outs:
        y.fill_(float("nan"))
    xd = x.cuda()
    y = stack.forward(xd, flags=(fc.FLAG_DENSE_K if mode == "dense" else 0), padded=(mode == "padded"),
                      compact=(mode == "compact"))
    torch.cuda.synchronize()
    assert not bool(torch.isnan(y).any()), "unwritten output elements"
    ref = oracle_chain(oracle, name, layers, x, ws, bs, images)
    got = f64(y[images])
    err = rel_l2_per_image(got, ref)
    print("config %s %s: rel-L2 = %.3e (tol %.1e)" % (name, mode, err, TOL[layers[0].dtype]), flush=True)
    assert err <= TOL[layers[0].dtype]
    # element by element, layer by layer, each layer fed what the GPU fed it
    a_in = f64(x[images])
    for i, (l, w, b, yo) in enumerate(zip(layers, ws, bs, stack.outs)):
        a_out = f64(yo[images])
        worst = check_layer_elementwise(oracle, l, a_in, w, b, a_out, "%s %s layer %d" % (name, mode, i + 1))
        print("  layer %d: worst element at %.2f of its bound" % (i + 1, worst), flush=True)
        a_in = a_out


def test_store_pacing_changes_nothing(env):
    """The headline layer at full size is long enough for the streaming kernels to pace their store
    bursts on the wall clock (its run against the oracle above is a paced one).  With
    FOLDCONV_FLAG_UNPACED the same bytes come out: folded path, zero-padded reference, channels-first
    output.  Several launches each, so that waves do sleep in the paced ones."""
    fc, runner, wl = env
    layers, x, ws, bs = wl.make_config("c2")
    l = layers[0]
    L = runner.FoldedLayer(l, ws[0], bs[0])
    xd = x.cuda()
    y_paced, y_free = L.new_output(), L.new_output()
    for _ in range(5):
        L.forward(xd, y_paced)
        L.forward(xd, y_free, flags=fc.FLAG_UNPACED)
    torch.cuda.synchronize()
    assert torch.equal(y_paced, y_free)
    # a paced launch replayed from a captured graph (it reads the wall clock, no host state): every replay, with
    # eager launches and synchronisations in between, writes the same bytes
    y_graph = L.new_output()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        L.forward(xd, y_graph)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        L.forward(xd, y_graph)
    for _ in range(3):
        y_graph.fill_(float("nan"))
        gr.replay()
        L.forward(xd, y_free, flags=fc.FLAG_UNPACED)
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_paced)
    del gr, y_graph
    for _ in range(3):
        L.forward_padded(xd, y_free)
    s = L.plan.shapes
    fc.conv_padded_forward(L.plan, xd, L.w, L.b, y_paced, L.ws_pad, fc.FLAG_FILTER_PACKED | fc.FLAG_UNPACED)
    torch.cuda.synchronize()
    assert torch.equal(y_paced, y_free)
    with pytest.raises(fc.FoldconvError) as e:    # the reference path still rejects flags it does not honour
        fc.conv_padded_forward(L.plan, xd, L.w, L.b, y_paced, L.ws_pad, fc.FLAG_DENSE_K)
    assert e.value.status == -1
    del y_paced, y_free
    # channels-first output from the same launch
    C = runner.ChannelsFirstLayer(l, ws[0].permute(3, 2, 0, 1).contiguous(), bs[0])
    assert C.fused and s.N == 64
    xc = x.permute(0, 3, 1, 2).contiguous().cuda()
    y1, y2 = C.new_output(), C.new_output()
    for _ in range(4):
        C.forward(xc, y1)
    flags = fc.FLAG_FILTER_PACKED | fc.FLAG_OUT_NCHW | fc.FLAG_UNPACED
    assert C.one_launch                           # the layer reads x channels-first in the same launch
    fc.foldconv_forward(C.plan, xc, C.w_exp, C.b, y2, C.ws, flags | fc.FLAG_IN_NCHW)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    fc.foldconv_fold_input_nchw(C.plan, xc, C.x_fold)     # ... and writes what the two-launch route writes
    fc.foldconv_forward(C.plan, C.x_fold, C.w_exp, C.b, y2, C.ws, flags)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)


def test_output_beyond_four_gigabytes(env, oracle):
    """Largest-size case: a tall-skinny product whose output (8.6 GB) needs more than 32 bits of
    byte offset, in the launch configuration the benchmark uses (packed filter, aliased fold).
    Rows are independent, so the oracle checks sampled row blocks from the start, the quarters,
    across the 4 GiB byte mark, and the end; every 16 Mi-th row block is also checked for
    unwritten elements."""
    fc, runner, wl = env
    M, K, N, F = 1 << 26, 8, 64, 4
    plan = fc.foldconv_plan_gemm(M, K, N, F, torch.float16)
    s = plan.shapes
    assert s.y_bytes == M * N * 2 >= (1 << 33) and s.conv_kernel == 2
    g = torch.Generator(device="cpu")
    g.manual_seed(4242)
    A = torch.randn((M, K), generator=g, dtype=torch.float32).to(torch.float16)
    B = (torch.randn((K, N), generator=g, dtype=torch.float32) / np.sqrt(K)).to(torch.float16)
    print("large gemm: inputs drawn", flush=True)
    xd, wd = A.cuda(), B.cuda()
    w_exp = torch.empty(s.w_exp_bytes // 2, dtype=torch.float16, device="cuda")
    fc.foldconv_expand_filter(plan, wd, w_exp)
    ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device="cuda")
    fc.foldconv_pack_filter(plan, w_exp, ws)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    fc.foldconv_fold_input(plan, xd, xd)
    fc.foldconv_forward(plan, xd, w_exp, None, y, ws, fc.FLAG_FILTER_PACKED)
    torch.cuda.synchronize()
    print("large gemm: kernel done", flush=True)
    rows_per_4g = (1 << 32) // (N * 2)
    assert rows_per_4g == M // 2
    starts = [0, M // 4 + 32, rows_per_4g - 64, 3 * (M // 4) - 32, M - 128]
    Bf = f64(B)
    for r0 in starts:
        got = f64(y[r0:r0 + 128].cpu())
        ref = oracle.conv_direct(f64(A[r0:r0 + 128]).reshape(1, 1, 128, K), Bf.reshape(1, 1, K, N), None, 0, 0)
        assert rel_l2_per_image(got.reshape(1, -1), ref.reshape(1, -1)) <= TOL["f16"], r0
    for r0 in range(0, M, 1 << 24):
        assert not bool(torch.isnan(y[r0:r0 + 4096]).any()), r0
    assert not bool(torch.isnan(y[-4096:]).any())


def test_stack_replays_from_a_captured_graph(env):
    """The library allocates nothing and never synchronises, so a whole stack of layers can be
    captured into a HIP graph.  Every replay (with eager work and synchronisations in between, and
    with new input data copied into the captured buffer) must reproduce the eager result bit for bit."""
    fc, runner, wl = env
    layers, x, ws, bs = wl.make_config("c5", N=2)
    stack = runner.FoldedStack(layers, ws, bs)
    xs = [x, torch.flip(x, dims=[2]).contiguous(), (x * 0.5).contiguous()]
    eager = []
    for xi in xs:
        y = stack.forward(xi.cuda())
        torch.cuda.synchronize()
        eager.append(y.clone())
    x_static = xs[0].cuda().clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        stack.forward(x_static)                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        y_static = stack.forward(x_static)
    for rep in range(2):
        for xi, want in zip(xs, eager):
            x_static.copy_(xi.cuda())
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y_static, want), rep
            y_static.add_(1.0)                       # eager work between replays; the next replay must overwrite it
