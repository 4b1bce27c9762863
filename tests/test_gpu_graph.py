"""The library's calls under HIP graph capture: they allocate nothing, do not synchronize and clear their
status words with kernels (no memset nodes), so a captured sequence must replay to the eager result every
time -- also after the inputs were rewritten in place and with other work between the replays."""
import numpy as np
import pytest

import wush_inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2512_00956_amd as P
    P.lib()
    return P


def _capture(fn):
    import torch
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        fn()                                    # warm-up outside the capture (one-time kernel attribute calls)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            fn()
    torch.cuda.synchronize()
    return g


@pytest.mark.parametrize("M", [16, 100, 700])
def test_layer_replays_to_the_eager_result(P, M):
    """Transform construction, weight preparation, activation quantizer and GEMM (plus the decode entry point
    for at most 64 tokens) in one graph; three replays on fresh activations."""
    import torch
    K, N = 1024, 1100
    gen = torch.Generator(device="cuda").manual_seed(100 + M)
    W = (torch.randn((N, K), device="cuda", generator=gen) * 0.05).to(torch.bfloat16)
    Xc = torch.randn((512, K), device="cuda", generator=gen).to(torch.bfloat16)
    X = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
    fmt = P.default_fmt(layout=1)
    T = torch.empty((K // 32, 32, 32), dtype=torch.bfloat16, device="cuda")
    bws = torch.empty(P.wush_build_transforms_workspace(K), dtype=torch.uint8, device="cuda")
    (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes(M, K, fmt), P.wush_packed_sizes(N, K, fmt)
    Xq, Xs = torch.empty(xcb, dtype=torch.uint8, device="cuda"), torch.empty(xsb, dtype=torch.uint8, device="cuda")
    Wq, Ws = torch.empty(wcb, dtype=torch.uint8, device="cuda"), torch.empty(wsb, dtype=torch.uint8, device="cuda")
    wsp = torch.empty(P.wush_prepare_weight_workspace(N, K), dtype=torch.uint8, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    Yd = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    Yst = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dws = torch.empty(P.wush_layer_decode_workspace(K), dtype=torch.uint8, device="cuda")
    P.wush_layer_decode_init(dws, K)

    def layer():
        P.wush_build_transforms(W, Xc, 1e-2, T, bws)
        P.wush_prepare_weight(W, T, Wq, Ws, wsp, fmt)
        P.wush_quantize_act(X, T, Xq, Xs, fmt)
        P.wush_linear(Xq, Xs, Wq, Ws, Y, fmt, K=K)
        if M <= 64:
            P.wush_layer_decode(X, T, Wq, Ws, Yd, dws, fmt)
            P.wush_layer_decode_static(X, T, Wq, Ws, Yst, fmt)     # staging in the library's static device array

    g = _capture(layer)
    for rep in range(3):
        X.copy_(torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16))   # new activations, same addresses
        T.zero_(); Y.fill_(float("nan")); Yd.fill_(float("nan")); Yst.fill_(float("nan")); Xq.zero_(); Wq.zero_()
        g.replay()
        torch.cuda.synchronize()
        got = (T.clone(), Wq.clone(), Ws.clone(), Xq.clone(), Xs.clone(), Y.clone(), Yd.clone(), Yst.clone())
        scratch = torch.randn((1 << 20,), device="cuda").sum().item()                     # unrelated eager work and a sync
        assert np.isfinite(scratch)
        layer()
        torch.cuda.synchronize()
        P.wush_workspace_status(wsp, K)
        for name, a, b in zip(("T", "Wq", "Ws", "Xq", "Xs", "Y", "Yd", "Yst"), got, (T, Wq, Ws, Xq, Xs, Y, Yd, Yst)):
            if name in ("Yd", "Yst") and M > 64:
                continue
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (rep, name)
        if M <= 64:
            assert torch.equal(Yd.view(torch.uint8), Yst.view(torch.uint8))
        assert not bool(Y.isnan().any())


@pytest.mark.parametrize("M", [300, 40])          # the tiled GEMM, and the weight-streaming one for few tokens
def test_nvfp4_and_int4_layers_replay_to_the_eager_result(P, M):
    import torch
    K, N = 1024, 520
    gen = torch.Generator(device="cuda").manual_seed(7)
    W = (torch.randn((N, K), device="cuda", generator=gen) * 0.05).to(torch.bfloat16)
    X = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
    T16 = torch.from_numpy(I.make_transforms_random(K // 16, 3, block=16).view(np.int16)).view(torch.bfloat16).cuda()
    T32 = torch.from_numpy(I.make_transforms_random(K // 32, 4).view(np.int16)).view(torch.bfloat16).cuda()
    (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, 1), P.wush_packed_sizes_nvfp4(N, K, 1)
    e = lambda n: torch.empty(n, dtype=torch.uint8, device="cuda")
    Xq, Xs, Wq, Ws = e(xcb), e(xsb), e(wcb), e(wsb)
    Xq4, Xs4, Wq4, Ws4 = e(xcb), e(xsb), e(wcb), e(wsb)
    tsx = torch.full((1,), 0.01, dtype=torch.float32, device="cuda")
    tsw = torch.zeros(1, dtype=torch.float32, device="cuda")
    wsn, wsi = e(P.wush_prepare_weight_nvfp4_workspace(K)), e(P.wush_prepare_weight_workspace(N, K))
    Yn = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    Yi = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")

    def layers():
        P.wush_prepare_weight_nvfp4(W, T16, Wq, Ws, tsw, wsn, layout=1)
        P.wush_quantize_act_nvfp4(X, T16, tsx, Xq, Xs, layout=1)
        P.wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Yn, layout=1, K=K)
        P.wush_prepare_weight_int4(W, T32, Wq4, Ws4, wsi, layout=1)
        P.wush_quantize_act_int4(X, T32, Xq4, Xs4, layout=1)
        P.wush_linear_int4(Xq4, Xs4, Wq4, Ws4, Yi, layout=1, K=K)

    g = _capture(layers)
    for rep in range(3):
        X.copy_(torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16))
        Yn.fill_(float("nan")); Yi.fill_(float("nan")); tsw.zero_()
        g.replay()
        torch.cuda.synchronize()
        got = (Yn.clone(), Yi.clone(), tsw.clone(), Xq.clone(), Xq4.clone())
        assert np.isfinite(torch.randn((1 << 20,), device="cuda").sum().item())
        layers()
        torch.cuda.synchronize()
        for name, a, b in zip(("Yn", "Yi", "tsw", "Xq", "Xq4"), got, (Yn, Yi, tsw, Xq, Xq4)):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (rep, name)
        assert not bool(Yn.isnan().any()) and not bool(Yi.isnan().any())
