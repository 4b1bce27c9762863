"""GPU parity of the NVFP4 variant (16 x 16 transforms, E2M1 elements, E4M3 scale per
16, FP32 tensor scale) against oracle/wush_nvfp4_oracle.py, through the C ABI.
Bars: quantizer bit-exact when both sides see the same FP32 values; transformed
values within 1e-5 of the group AbsMax; codes against the all-FP64 path differ only
next to a decision boundary; GEMM relative Frobenius error <= 2e-3 (BF16 output) and
<= 1e-5 (FP32 output)."""
import numpy as np
import pytest

import wush_inputs as I
from oracle import wush_nvfp4_oracle as NV
from oracle import wush_oracle as O
from tests import kernel_models as KM

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2512_00956_amd as P
    P.lib()
    return P


def _force_width(P, width):
    """Force the tile width of the tiled GEMM and keep the weight-streaming kernel out of the way."""
    P.wush_debug_set(P.WUSH_DEBUG_W4_WIDTH, int(width))
    P.wush_debug_set(P.WUSH_DEBUG_W4_SKINNY, 0)


@pytest.fixture(autouse=True)
def _reset_switches(P):
    yield
    P.wush_debug_set(P.WUSH_DEBUG_W4_WIDTH, -1)
    P.wush_debug_set(P.WUSH_DEBUG_W4_SKINNY, -1)


@pytest.fixture(scope="module")
def G():
    from tests import gpu_util
    return gpu_util


def _f32_dev(x):
    import torch
    return torch.tensor([float(x)], dtype=torch.float32, device="cuda")


def _wush16(W, Xc, lam=1e-2):
    K = W.shape[1]
    T = np.empty((K // 16, 16, 16))
    for b in range(K // 16):
        sl = slice(16 * b, 16 * b + 16)
        T[b] = O.wush_block(O.second_moment(W[:, sl]), O.second_moment(Xc[:, sl]), lam)
    return O.round_to_bf16(T)


SHAPES = {
    "c1": I.CONFIGS["c1"],
    "ragged": I.scaled(I.CONFIGS["c1"], M=77, K=32 * 13, N=45, calib_tokens=256, n_outlier=3),
    "tiles": I.scaled(I.CONFIGS["c2"], M=300, K=1024, N=520, calib_tokens=1024, n_outlier=5),
    "one_token": I.scaled(I.CONFIGS["c1"], M=1, K=128, N=32, calib_tokens=256, n_outlier=1),
}
_cache = {}


def _layer(name):
    if name not in _cache:
        cfg = SHAPES[name]
        L = I.make_layer(cfg)
        X, Xc, W = (O.bf16_bits_to_f64(L[k]) for k in ("X", "X_cal", "W"))
        _cache[name] = (cfg, L, X, W, _wush16(W, Xc))
    return _cache[name]


def _pack(codes):
    return O.pack_codes(codes)


def _adversarial_groups():
    """Groups on every E2M1 midpoint, with AbsMax on E4M3 midpoints and thresholds."""
    pts = []
    for mpt in (0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0):
        f = np.float32(mpt)
        pts += [f, -np.nextafter(f, np.float32(0)), np.nextafter(f, np.float32(10))]
    pts = np.array(pts[:15], dtype=np.float32)
    rows = []
    grid = NV.e4m3_value(np.arange(127))
    mids = ((grid[1:] + grid[:-1]) / 2)[::7]
    for top in list(mids) + [448.0, 464.0, 500.0, 2.0 ** -10, 2.0 ** -9, 3 * 2.0 ** -10, 1e-4, 0.0]:
        g = np.zeros(16, dtype=np.float32)
        g[:15] = pts * np.float32(top / 6.0 if top > 0 else 0.0)
        g[15] = -np.float32(6.0 * top)
        rows.append(g)
    z = np.zeros(16, dtype=np.float32)
    z[2] = -0.0
    rows.append(z)
    return np.stack(rows)


@pytest.mark.parametrize("ts", [1.0, 0.0123, 3.7e-5])
def test_quantizer_tap_bit_exact(P, G, ts):
    import torch
    adv = _adversarial_groups() * np.float32(ts)
    rnd = I.random_f32((257, 16 * 9), seed=12, spread=6.0) * np.float32(ts)
    pad = (-adv.shape[0]) % 9
    adv = np.concatenate([adv, np.zeros((pad, 16), np.float32)]).reshape(-1, 16 * 9)
    Y = np.concatenate([rnd, adv]).astype(np.float32)
    # rows must be a multiple of 32 channels wide for the entry point: 144 = 4.5 * 32 -> widen to 288
    Y = np.concatenate([Y, Y[::-1]], axis=1)
    M, K = Y.shape
    q, s = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_quantize_f32_nvfp4(torch.from_numpy(Y).cuda(), _f32_dev(ts), q, s)
    torch.cuda.synchronize()
    # the kernel does exactly the steps it states (bit for bit) ...
    cr, sr = KM.nvfp4_steps(Y, np.float32(ts), np.float32)
    assert np.array_equal(G.host(s), sr)
    assert np.array_equal(G.host(q), _pack(cr))
    # ... and those steps differ from the definition (FP64, true divisions) only next to a rounding boundary
    cd, sd = NV.quantize_nvfp4(Y, np.float32(ts))
    rate, unexplained = KM.nvfp4_explained(Y.astype(np.float64), np.float32(ts), cr, sr, cd, sd, tol=1e-6)
    assert unexplained == 0, (rate, unexplained)


def test_quantizer_tap_zero_tensor_scale(P, G):
    import torch
    Y = I.random_f32((4, 64), seed=3, spread=2.0)
    q, s = G.empty_u8(4, 32), G.empty_u8(4, 4)
    P.wush_quantize_f32_nvfp4(torch.from_numpy(Y).cuda(), _f32_dev(0.0), q, s)
    torch.cuda.synchronize()
    cr, sr = NV.quantize_nvfp4(Y, 0.0)       # no arithmetic left to model: the definition itself
    assert not sr.any() and np.array_equal(G.host(s), sr) and np.array_equal(G.host(q), _pack(cr))


@pytest.mark.parametrize("name", list(SHAPES))
def test_transform_quant(P, G, name):
    import torch
    cfg, L, X, W, T = _layer(name)
    M, K = cfg.M, cfg.K
    Yt = NV.transform_act(X, T)
    ts = NV.tensor_scale(Yt)
    Xd, Td = G.bf16_dev(L["X"]), G.bf16_dev(O.bf16_values_to_bits(T))
    Xq, Xs = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    dbg = torch.full((M, K), float("nan"), dtype=torch.float32, device="cuda")
    P.wush_quantize_act_nvfp4(Xd, Td, _f32_dev(ts), Xq, Xs, dbg_Yt=dbg)
    Xq2, Xs2 = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_quantize_act_nvfp4(Xd, Td, _f32_dev(ts), Xq2, Xs2)
    torch.cuda.synchronize()
    xq, xs, yt = G.host(Xq), G.host(Xs), G.host(dbg)
    assert np.array_equal(xq, G.host(Xq2)) and np.array_equal(xs, G.host(Xs2))
    # (1) quantizer bit-exact on the kernel's own FP32 values
    assert np.isfinite(yt).all()
    cr, sr = KM.nvfp4_steps(yt, ts, np.float32)
    assert np.array_equal(xs, sr)
    assert np.array_equal(xq, _pack(cr))
    # (2) transformed values against FP64
    amax = np.max(np.abs(Yt.reshape(M, K // 16, 16)), axis=-1)
    err = np.max(np.abs(yt.astype(np.float64) - Yt).reshape(M, K // 16, 16), axis=-1)
    assert np.max(err / amax) <= 1e-5
    # (3) codes against the all-FP64 path: differences only next to a decision boundary
    c64, s64 = NV.quantize_nvfp4(Yt, ts)
    rate, unexplained = KM.nvfp4_explained(Yt, ts, O.unpack_codes(xq), xs, c64, s64, tol=1e-5)
    assert rate <= 2e-4 and unexplained == 0, (rate, unexplained)


@pytest.mark.parametrize("name", list(SHAPES))
def test_calibrate_act(P, G, name):
    """AbsMax of T X / (6 * 448) on the device against the oracle's (FP32 accumulators against FP64)."""
    import torch
    cfg, L, X, W, T = _layer(name)
    ts = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    P.wush_calibrate_act_nvfp4(G.bf16_dev(L["X"]), G.bf16_dev(O.bf16_values_to_bits(T)), ts)
    torch.cuda.synchronize()
    ref = float(NV.tensor_scale(NV.transform_act(X, T)))
    assert abs(float(ts.cpu()[0]) - ref) <= 1e-5 * ref
    # a second call on the same word starts from zero again
    P.wush_calibrate_act_nvfp4(G.bf16_dev(L["X"][:1]), G.bf16_dev(O.bf16_values_to_bits(T)), ts)
    torch.cuda.synchronize()
    ref1 = float(NV.tensor_scale(NV.transform_act(X[:1], T)))
    assert abs(float(ts.cpu()[0]) - ref1) <= 1e-5 * ref1


def test_transform_quant_is_independent_of_the_launch_shape(P, G):
    """A large, ragged batch (workgroups of two wave groups, nine tiles each, a last tile of three tokens)
    gives, row for row, the bytes the same rows give in small batches, in both layouts."""
    import torch
    M, K = 4099, 8192
    X = torch.from_numpy(I.random_f32((M, K), seed=42, spread=2.0)).cuda().to(torch.bfloat16)
    T = G.bf16_dev(I.make_transforms_random(K // 16, 4, block=16))
    ts = _f32_dev(0.01)
    Xq, Xs = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_quantize_act_nvfp4(X, T, ts, Xq, Xs)
    cb, sb = P.wush_packed_sizes_nvfp4(M, K, 1)
    Xqt, Xst = G.empty_u8(cb), G.empty_u8(sb)
    P.wush_quantize_act_nvfp4(X, T, ts, Xqt, Xst, layout=1)
    Xqu, Xsu = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_unpack_tiled_nvfp4(Xqt, Xst, M, K, Xqu, Xsu)
    torch.cuda.synchronize()
    assert torch.equal(Xqu, Xq) and torch.equal(Xsu, Xs)
    for lo, hi in ((0, 256), (1500, 1533), (4064, 4099)):
        q, s_ = G.empty_u8(hi - lo, K // 2), G.empty_u8(hi - lo, K // 16)
        P.wush_quantize_act_nvfp4(X[lo:hi], T, ts, q, s_)
        torch.cuda.synchronize()
        assert torch.equal(q, Xq[lo:hi]) and torch.equal(s_, Xs[lo:hi]), (lo, hi)


def test_transform_quant_strided_rows(P, G):
    import torch
    cfg, L, X, W, T = _layer("ragged")
    M, K = cfg.M, cfg.K
    ts = _f32_dev(NV.tensor_scale(NV.transform_act(X, T)))
    wide = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda")
    wide[:, :K] = G.bf16_dev(L["X"])
    Td = G.bf16_dev(O.bf16_values_to_bits(T))
    Xq, Xs = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    Xq2, Xs2 = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_quantize_act_nvfp4(wide[:, :K], Td, ts, Xq, Xs)
    P.wush_quantize_act_nvfp4(G.bf16_dev(L["X"]), Td, ts, Xq2, Xs2)
    torch.cuda.synchronize()
    assert np.array_equal(G.host(Xq), G.host(Xq2)) and np.array_equal(G.host(Xs), G.host(Xs2))


@pytest.mark.parametrize("name", list(SHAPES))
def test_prepare_weight(P, G, name):
    import torch
    cfg, L, X, W, T = _layer(name)
    N, K = cfg.N, cfg.K
    Wd, Td = G.bf16_dev(L["W"]), G.bf16_dev(O.bf16_values_to_bits(T))
    Wq, Ws = G.empty_u8(N, K // 2), G.empty_u8(N, K // 16)
    tsw = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = G.empty_u8(P.wush_prepare_weight_nvfp4_workspace(K))
    P.wush_prepare_weight_nvfp4(Wd, Td, Wq, Ws, tsw, ws)
    P.wush_prepare_weight_nvfp4_status(ws, K)
    cr, sr, ts_ref = NV.prepare_weight(W, T)
    ts_gpu = np.float32(tsw.cpu().numpy()[0])
    assert abs(float(ts_gpu) - float(ts_ref)) <= 1.2e-7 * float(ts_ref)      # at most one FP32 ulp
    Wt = NV.transform_weight(W, T)
    if ts_gpu != ts_ref:
        cr, sr = NV.quantize_nvfp4(Wt, ts_gpu)
    rate, unexplained = KM.nvfp4_explained(Wt, ts_gpu, O.unpack_codes(G.host(Wq)), G.host(Ws), cr, sr, tol=1e-9)
    assert rate <= 1e-4 and unexplained == 0, (rate, unexplained)


def test_prepare_weight_flags_singular_block(P, G):
    import torch
    K, N = 64, 40
    T = np.stack([np.eye(16)] * 4)
    T[2, 5, :] = 0.0                                   # rank-deficient third block
    Wd = G.bf16_dev(I.f32_to_bf16_bits(I.random_f32((N, K), 5, 1.0)))
    Wq, Ws = G.empty_u8(N, K // 2), G.empty_u8(N, K // 16)
    tsw = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = G.empty_u8(P.wush_prepare_weight_nvfp4_workspace(K))
    P.wush_prepare_weight_nvfp4(Wd, G.bf16_dev(O.bf16_values_to_bits(T)), Wq, Ws, tsw, ws)
    with pytest.raises(P.WushError) as e:
        P.wush_prepare_weight_nvfp4_status(ws, K)
    assert e.value.code == 7
    # a good tensor clears the flag again
    P.wush_prepare_weight_nvfp4(Wd, G.bf16_dev(O.bf16_values_to_bits(np.stack([np.eye(16)] * 4))), Wq, Ws, tsw, ws)
    P.wush_prepare_weight_nvfp4_status(ws, K)


GEMM_SHAPES = [(16, 256, 64), (77, 45, 128), (300, 520, 192), (257, 256, 1024), (512, 768, 4096), (1, 32, 256)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_linear_against_oracle(P, G, M, N, K, out):
    """GEMM alone: both sides start from the same codes, scale bytes and tensor scales."""
    import torch
    rng = np.random.default_rng(1000 + M + N + K)
    xc = rng.integers(0, 16, (M, K), dtype=np.uint8)
    wc = rng.integers(0, 16, (N, K), dtype=np.uint8)
    xs = rng.integers(0, 127, (M, K // 16), dtype=np.uint8)       # every finite E4M3 byte, subnormals included
    ws_ = rng.integers(40, 80, (N, K // 16), dtype=np.uint8)
    tsx, tsw = np.float32(0.0371), np.float32(2.4e-4)
    ref = NV.linear_dequant(xc, xs, tsx, wc, ws_, tsw)
    f32 = out == "f32"
    Y = torch.full((M, N + 8), float("nan"), dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")
    P.wush_linear_nvfp4(G.u8_dev(_pack(xc)), G.u8_dev(xs), _f32_dev(tsx), G.u8_dev(_pack(wc)), G.u8_dev(ws_),
                        _f32_dev(tsw), Y[:, :N], out_dtype=1 if f32 else 0)
    torch.cuda.synchronize()
    y = Y.float().cpu().numpy().astype(np.float64)
    assert np.isnan(y[:, N:]).all()                      # nothing written past N
    assert O.rel_fro(y[:, :N], ref) <= (1e-5 if f32 else 2e-3)


def _tile_operand(packed, scales):
    """Canonical packed codes [rows][K/2] and scale bytes [rows][K/16] -> the tiled buffers, from the
    statement of the layout: rows padded to 32; the 16-byte chunk (row, kt, hh) of a 64-element K step at
    ((((row / 32) KT + kt) 2 + hh) 32 + row % 32) 16, the scale dword (row, kt) at (((row / 32) KT + kt) 32 + row % 32) 4."""
    rows, K = packed.shape[0], packed.shape[1] * 2
    KT, RB = K // 64, (rows + 31) // 32
    q = np.zeros((RB, KT, 2, 32, 16), dtype=np.uint8)
    sc = np.zeros((RB, KT, 32, 4), dtype=np.uint8)
    pq = np.zeros((RB * 32, KT, 2, 16), dtype=np.uint8)
    pq[:rows] = packed.reshape(rows, KT, 2, 16)
    ps = np.zeros((RB * 32, KT, 4), dtype=np.uint8)
    ps[:rows] = scales.reshape(rows, KT, 4)
    q[:] = pq.reshape(RB, 32, KT, 2, 16).transpose(0, 2, 3, 1, 4)
    sc[:] = ps.reshape(RB, 32, KT, 4).transpose(0, 2, 1, 3)
    return q.reshape(-1), sc.reshape(-1)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("K", [320, 384])
@pytest.mark.parametrize("width", ["2", "3", "4"])
def test_linear_every_tile_width(P, G, width, K, layout):
    """The three tile widths (128, 192, 256 output channels) on a shape with several tiles and ragged
    edges in both directions; the library normally chooses by cost.  An odd number of 64-element K
    steps (K = 320) takes the kernel that stages both operands in LDS, an even one (K = 384) the one
    that keeps W in registers; both read either layout."""
    import torch
    _force_width(P, width)
    M, N = 300, 700
    rng = np.random.default_rng(77 + K)
    xc = rng.integers(0, 16, (M, K), dtype=np.uint8)
    wc = rng.integers(0, 16, (N, K), dtype=np.uint8)
    xs = rng.integers(30, 100, (M, K // 16), dtype=np.uint8)
    ws_ = rng.integers(0, 127, (N, K // 16), dtype=np.uint8)
    tsx, tsw = np.float32(1.7), np.float32(3.1e-3)
    ref = NV.linear_dequant(xc, xs, tsx, wc, ws_, tsw)
    Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    xq, wq = _pack(xc), _pack(wc)
    if layout:
        (xq, xs), (wq, ws_) = _tile_operand(xq, xs), _tile_operand(wq, ws_)
    P.wush_linear_nvfp4(G.u8_dev(xq), G.u8_dev(xs), _f32_dev(tsx), G.u8_dev(wq), G.u8_dev(ws_), _f32_dev(tsw), Y,
                        layout=layout, out_dtype=1, K=K)
    torch.cuda.synchronize()
    assert O.rel_fro(Y.cpu().numpy().astype(np.float64), ref) <= 1e-5


@pytest.mark.parametrize("kernel", [1, 2, 0, -1], ids=["streaming_split_k", "streaming_shared_x", "tiled", "library_choice"])
@pytest.mark.parametrize("M", [1, 2, 7, 16, 31, 32, 33, 48, 64, 65, 100, 128])
@pytest.mark.parametrize("K", [64, 320, 1024])
def test_linear_few_tokens_on_either_kernel(P, G, K, M, kernel):
    """Up to 128 tokens the tiled layout takes a weight-streaming kernel (one workgroup per 32 output
    channels, K split over its four waves; beyond 64 tokens also one workgroup per 128 output channels whose
    waves share the converted activations through LDS); they and the tiled kernel are forced in turn on a ragged
    shape, FP32 and BF16 output, against the oracle on the same codes, scales and tensor scales."""
    import torch
    N = 1000
    rng = np.random.default_rng(4000 + 7 * M + K)
    xc = rng.integers(0, 16, (M, K), dtype=np.uint8)
    wc = rng.integers(0, 16, (N, K), dtype=np.uint8)
    xs = rng.integers(0, 127, (M, K // 16), dtype=np.uint8)
    ws_ = rng.integers(40, 100, (N, K // 16), dtype=np.uint8)
    tsx, tsw = np.float32(0.0371), np.float32(2.4e-4)
    ref = NV.linear_dequant(xc, xs, tsx, wc, ws_, tsw)
    (xq, xst), (wq, wst) = _tile_operand(_pack(xc), xs), _tile_operand(_pack(wc), ws_)
    P.wush_debug_set(P.WUSH_DEBUG_W4_SKINNY, kernel)
    for f32 in (True, False):
        Y = torch.full((M, N + 8), float("nan"), dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")
        P.wush_linear_nvfp4(G.u8_dev(xq), G.u8_dev(xst), _f32_dev(tsx), G.u8_dev(wq), G.u8_dev(wst), _f32_dev(tsw),
                            Y[:, :N], layout=1, out_dtype=1 if f32 else 0, K=K)
        torch.cuda.synchronize()
        y = Y.float().cpu().numpy().astype(np.float64)
        assert np.isnan(y[:, N:]).all()
        assert np.isfinite(y[:, :N]).all()
        assert O.rel_fro(y[:, :N], ref) <= (1e-5 if f32 else 2e-3), (f32, O.rel_fro(y[:, :N], ref))


@pytest.mark.parametrize("name", ["c1", "tiles"])
def test_layer_end_to_end(P, G, name):
    import torch
    cfg, L, X, W, T = _layer(name)
    M, N, K = cfg.M, cfg.N, cfg.K
    if K % 64:
        pytest.skip("GEMM needs K % 64 == 0")
    Yt = NV.transform_act(X, T)
    ts = NV.tensor_scale(Yt)
    Xd, Wd, Td = G.bf16_dev(L["X"]), G.bf16_dev(L["W"]), G.bf16_dev(O.bf16_values_to_bits(T))
    Xq, Xs = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    Wq, Ws = G.empty_u8(N, K // 2), G.empty_u8(N, K // 16)
    tsx, tsw = _f32_dev(ts), torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = G.empty_u8(P.wush_prepare_weight_nvfp4_workspace(K))
    P.wush_prepare_weight_nvfp4(Wd, Td, Wq, Ws, tsw, ws)
    P.wush_quantize_act_nvfp4(Xd, Td, tsx, Xq, Xs)
    Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    P.wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Y, out_dtype=1)
    torch.cuda.synchronize()
    ref = NV.layer_forward(X, W, T, tsx=ts)
    # a handful of boundary codes may differ; their effect on the output is far below the bar
    assert O.rel_fro(Y.cpu().numpy().astype(np.float64), ref) <= 2e-3
    # and the quantized layer approximates the unquantized product as the oracle's does
    exact = X @ W.T
    assert abs(O.rel_fro(Y.cpu().numpy().astype(np.float64), exact) - O.rel_fro(ref, exact)) <= 1e-3


def test_tiled_layout_is_a_permutation_of_canonical(P, G):
    """Both quantizers and the tap write the tiled layout; unpacking it gives the canonical bytes."""
    import torch
    cfg, L, X, W, T = _layer("tiles")
    M, N, K = cfg.M, cfg.N, cfg.K
    ts = _f32_dev(NV.tensor_scale(NV.transform_act(X, T)))
    Xd, Wd, Td = G.bf16_dev(L["X"]), G.bf16_dev(L["W"]), G.bf16_dev(O.bf16_values_to_bits(T))
    for rows, run in ((M, "act"), (N, "weight"), (M, "tap")):
        cb, sb = P.wush_packed_sizes_nvfp4(rows, K, 1)
        assert cb == (rows + 31) // 32 * 32 * K // 2 and sb == (rows + 31) // 32 * 32 * K // 16
        qt = torch.full((cb,), 0xEE, dtype=torch.uint8, device="cuda")
        st = torch.full((sb,), 0xEE, dtype=torch.uint8, device="cuda")
        qc, sc = G.empty_u8(rows, K // 2), G.empty_u8(rows, K // 16)
        if run == "act":
            P.wush_quantize_act_nvfp4(Xd, Td, ts, qt, st, layout=1)
            P.wush_quantize_act_nvfp4(Xd, Td, ts, qc, sc)
        elif run == "weight":
            tsw = torch.zeros(1, dtype=torch.float32, device="cuda")
            ws = G.empty_u8(P.wush_prepare_weight_nvfp4_workspace(K))
            P.wush_prepare_weight_nvfp4(Wd, Td, qt, st, tsw, ws, layout=1)
            P.wush_prepare_weight_nvfp4(Wd, Td, qc, sc, tsw, ws)
        else:
            Y = torch.from_numpy(I.random_f32((rows, K), seed=5, spread=3.0)).cuda()
            P.wush_quantize_f32_nvfp4(Y, ts, qt, st, layout=1)
            P.wush_quantize_f32_nvfp4(Y, ts, qc, sc)
        qu, su = G.empty_u8(rows, K // 2), G.empty_u8(rows, K // 16)
        P.wush_unpack_tiled_nvfp4(qt, st, rows, K, qu, su)
        torch.cuda.synchronize()
        assert np.array_equal(G.host(qu), G.host(qc)), run
        assert np.array_equal(G.host(su), G.host(sc)), run
        # an independent statement of the layout: chunk (row, kt, hh) and scale dword (row, kt)
        qh, sh, qch, sch = G.host(qt), G.host(st), G.host(qc), G.host(sc)
        KT = K // 64
        for row, kt, hh in ((0, 0, 0), (rows - 1, KT - 1, 1), (min(37, rows - 1), 3, 1), (rows // 2, 5, 0)):
            off = ((((row // 32) * KT + kt) * 2 + hh) * 32 + row % 32) * 16
            assert np.array_equal(qh[off:off + 16], qch[row, kt * 32 + hh * 16: kt * 32 + hh * 16 + 16])
            so = (((row // 32) * KT + kt) * 32 + row % 32) * 4
            assert np.array_equal(sh[so:so + 4], sch[row, kt * 4: kt * 4 + 4])


@pytest.mark.parametrize("width", ["2", "3", "4"])
def test_layer_end_to_end_tiled(P, G, width):
    """The path the benchmark times: tiled buffers from both quantizers into the GEMM."""
    import torch
    _force_width(P, width)
    cfg, L, X, W, T = _layer("tiles")
    M, N, K = cfg.M, cfg.N, cfg.K
    Yt = NV.transform_act(X, T)
    ts = NV.tensor_scale(Yt)
    Xd, Wd, Td = G.bf16_dev(L["X"]), G.bf16_dev(L["W"]), G.bf16_dev(O.bf16_values_to_bits(T))
    xcb, xsb = P.wush_packed_sizes_nvfp4(M, K, 1)
    wcb, wsb = P.wush_packed_sizes_nvfp4(N, K, 1)
    Xq, Xs, Wq, Ws = G.empty_u8(xcb), G.empty_u8(xsb), G.empty_u8(wcb), G.empty_u8(wsb)
    tsx, tsw = _f32_dev(ts), torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = G.empty_u8(P.wush_prepare_weight_nvfp4_workspace(K))
    P.wush_prepare_weight_nvfp4(Wd, Td, Wq, Ws, tsw, ws, layout=1)
    P.wush_quantize_act_nvfp4(Xd, Td, tsx, Xq, Xs, layout=1)
    Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    P.wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Y, layout=1, out_dtype=1, K=K)
    # the same through the canonical layout: identical accumulation order, identical bits
    Xq2, Xs2, Wq2, Ws2 = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16), G.empty_u8(N, K // 2), G.empty_u8(N, K // 16)
    P.wush_prepare_weight_nvfp4(Wd, Td, Wq2, Ws2, tsw, ws)
    P.wush_quantize_act_nvfp4(Xd, Td, tsx, Xq2, Xs2)
    Y2 = torch.empty((M, N), dtype=torch.float32, device="cuda")
    P.wush_linear_nvfp4(Xq2, Xs2, tsx, Wq2, Ws2, tsw, Y2, out_dtype=1)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)
    assert O.rel_fro(Y.cpu().numpy().astype(np.float64), NV.layer_forward(X, W, T, tsx=ts)) <= 2e-3


@pytest.mark.parametrize("name", ["c2", "c5"])
def test_bench_shapes_full_size(P, G, name):
    """The configurations bench.py times for the workloads n2 (2048 x 4096 -> 6144) and n5 (8192 x 8192 ->
    57344), tiled layout, BF16 output: sampled token rows, weight rows and output entries against the oracle."""
    import torch
    L = I.make_layer(I.CONFIGS[name])
    cfg = L["cfg"]
    M, K, N = cfg.M, cfg.K, cfg.N
    T = np.empty((K // 16, 16, 16))
    for b in range(K // 16):
        sl = slice(16 * b, 16 * b + 16)
        T[b] = O.wush_block(O.second_moment(O.bf16_bits_to_f64(L["W"][:, sl])),
                            O.second_moment(O.bf16_bits_to_f64(L["X_cal"][:, sl])), 1e-2)
    T = O.round_to_bf16(T)
    rng = np.random.default_rng(22)
    rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, 48)]))
    cols = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, 256)]))
    X = O.bf16_bits_to_f64(L["X"][rows])
    Yt = NV.transform_act(X, T)
    ts = np.float32(np.max(np.abs(Yt)) / 2688.0 * 1.5)      # a calibrated constant, not the exact batch maximum
    Xd, Wd, Td = G.bf16_dev(L["X"]), G.bf16_dev(L["W"]), G.bf16_dev(O.bf16_values_to_bits(T))
    (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, 1), P.wush_packed_sizes_nvfp4(N, K, 1)
    Xq, Xs, Wq, Ws = G.empty_u8(xcb), G.empty_u8(xsb), G.empty_u8(wcb), G.empty_u8(wsb)
    tsx, tsw = _f32_dev(ts), torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = G.empty_u8(P.wush_prepare_weight_nvfp4_workspace(K))
    P.wush_prepare_weight_nvfp4(Wd, Td, Wq, Ws, tsw, ws, layout=1)
    P.wush_prepare_weight_nvfp4_status(ws, K)
    P.wush_quantize_act_nvfp4(Xd, Td, tsx, Xq, Xs, layout=1)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Y, layout=1, K=K)
    Xqc, Xsc, Wqc, Wsc = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16), G.empty_u8(N, K // 2), G.empty_u8(N, K // 16)
    P.wush_unpack_tiled_nvfp4(Xq, Xs, M, K, Xqc, Xsc)
    P.wush_unpack_tiled_nvfp4(Wq, Ws, N, K, Wqc, Wsc)
    torch.cuda.synchronize()
    assert not bool(Y.isnan().any())
    # activation rows against the all-FP64 path
    xq, xs = Xqc[rows.tolist()].cpu().numpy(), Xsc[rows.tolist()].cpu().numpy()
    c64, s64 = NV.quantize_nvfp4(Yt, ts)
    rate, unexplained = KM.nvfp4_explained(Yt, ts, O.unpack_codes(xq), xs, c64, s64, tol=1e-5)
    assert rate <= 2e-4 and unexplained == 0, ("activation codes", rate, unexplained)
    # weight rows (= output columns): the tensor scale needs the whole tensor, so take the GPU's
    # (checked against the oracle's on the small shapes) and verify it bounds the sampled rows
    ts_w = np.float32(tsw.cpu().numpy()[0])
    Wt = NV.transform_weight(O.bf16_bits_to_f64(L["W"][cols]), T)
    assert np.max(np.abs(Wt)) <= float(ts_w) * 2688.0 * (1 + 1e-6)
    cw, sw = NV.quantize_nvfp4(Wt, ts_w)
    wq, wsb_ = Wqc[cols.tolist()].cpu().numpy(), Wsc[cols.tolist()].cpu().numpy()
    rate, unexplained = KM.nvfp4_explained(Wt, ts_w, O.unpack_codes(wq), wsb_, cw, sw, tol=1e-9)
    assert rate <= 1e-4 and unexplained == 0, ("weight codes", rate, unexplained)
    # output entries: the GEMM on the GPU's own codes, and the oracle's whole forward
    y = O.bf16_bits_to_f64(G.host(Y[rows.tolist()][:, cols.tolist()].contiguous()))
    own = NV.linear_dequant(O.unpack_codes(xq), xs, ts, O.unpack_codes(wq), wsb_, ts_w)
    assert O.rel_fro(y, own) <= 2e-3
    ref = NV.linear_dequant(c64, s64, ts, cw, sw, ts_w)
    exact = X @ O.bf16_bits_to_f64(L["W"][cols]).T
    q_err = O.rel_fro(ref, exact)
    assert O.rel_fro(y, ref) <= max(2e-3, 0.05 * q_err) and q_err < 0.25, (O.rel_fro(y, ref), q_err)
    # every output tile: FP32 output, one seeded token row per band of 128 rows (the kernel's tiles are 256 rows
    # high) x ALL N columns against the dequantized FP64 product of the GPU's own codes (exact inputs, so FP32
    # accumulation and the FP32 tensor-scale multiply are the only differences), and BF16 == RNE(FP32) bit for bit
    Y32 = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    P.wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Y32, layout=1, out_dtype=1, K=K)
    torch.cuda.synchronize()
    assert not bool(Y32.isnan().any())
    band = np.array([min(b + int(rng.integers(0, 128)), M - 1) for b in range(0, M, 128)])
    y32 = Y32[band.tolist()].cpu().numpy()
    del Y32
    assert np.array_equal(G.host(Y[band.tolist()].contiguous()), O.bf16_values_to_bits(O.round_to_bf16(y32.astype(np.float64))))
    xc_b, xs_b = O.unpack_codes(Xqc[band.tolist()].cpu().numpy()), Xsc[band.tolist()].cpu().numpy()
    xn = np.linalg.norm(NV.dequantize_nvfp4(xc_b, xs_b, ts), axis=1)
    wq_host, ws_host = Wqc.cpu().numpy(), Wsc.cpu().numpy()

    def chunk(c0, width=2048):
        c1 = min(N, c0 + width)
        wc = O.unpack_codes(wq_host[c0:c1])
        part = NV.linear_dequant(xc_b, xs_b, ts, wc, ws_host[c0:c1], ts_w)
        d = y32[:, c0:c1].astype(np.float64) - part
        wn = np.linalg.norm(NV.dequantize_nvfp4(wc, ws_host[c0:c1], ts_w), axis=1)
        return float(np.sum(d * d)), float(np.sum(part * part)), float(np.max(np.abs(d) / (xn[:, None] * wn[None, :] + 1e-300)))

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=8) as ex:
        parts = list(ex.map(chunk, range(0, N, 2048)))
    num, den, worst = sum(q[0] for q in parts), sum(q[1] for q in parts), max(q[2] for q in parts)
    print(f"nvfp4 {name}: every-tile check on {len(band)} rows x {N} columns: rel. Frobenius {np.sqrt(num / den):.2e}, "
          f"largest element error / (|x| |w|) {worst:.2e}")
    assert np.sqrt(num / den) <= 1e-5 and worst <= 1e-5
    # the same weights through the kernels for few tokens (16: K split over the waves, the shape bench.py times as
    # dn2 / dn5; 100: activations shared through LDS on the wide layer), every output element, FP32 output
    for m in (16, 100):
        (mcb, msb) = P.wush_packed_sizes_nvfp4(m, K, 1)
        xq_m, xs_m = G.empty_u8(mcb), G.empty_u8(msb)
        P.wush_quantize_act_nvfp4(Xd[:m], Td, tsx, xq_m, xs_m, layout=1)
        Ym = torch.full((m, N), float("nan"), dtype=torch.float32, device="cuda")
        P.wush_linear_nvfp4(xq_m, xs_m, tsx, Wq, Ws, tsw, Ym, layout=1, out_dtype=1, K=K)
        torch.cuda.synchronize()
        y32 = Ym.cpu().numpy()
        assert np.isfinite(y32).all()
        xc_b, xs_b = O.unpack_codes(Xqc[:m].cpu().numpy()), Xsc[:m].cpu().numpy()     # rows of a batch do not depend on its size
        xn = np.linalg.norm(NV.dequantize_nvfp4(xc_b, xs_b, ts), axis=1)
        with ThreadPoolExecutor(max_workers=8) as ex:
            parts = list(ex.map(chunk, range(0, N, 2048)))
        num, den, worst = sum(q[0] for q in parts), sum(q[1] for q in parts), max(q[2] for q in parts)
        print(f"nvfp4 {name}, {m} tokens: rel. Frobenius {np.sqrt(num / den):.2e}, largest element error / (|x| |w|) {worst:.2e}")
        assert np.sqrt(num / den) <= 1e-5 and worst <= 1e-5


def test_argument_validation(P, G):
    import torch
    Xq, Xs = G.empty_u8(4, 48), G.empty_u8(4, 6)     # K = 96: not a multiple of 64
    Y = torch.empty((4, 4), dtype=torch.bfloat16, device="cuda")
    one = _f32_dev(1.0)
    with pytest.raises(P.WushError) as e:
        P.wush_linear_nvfp4(Xq, Xs, one, Xq, Xs, one, Y)
    assert e.value.code == 2
    with pytest.raises(P.WushError) as e:
        P.wush_linear_nvfp4(G.empty_u8(4, 64), G.empty_u8(4, 8), None, G.empty_u8(4, 64), G.empty_u8(4, 8), one, Y)
    assert e.value.code == 1
    with pytest.raises(P.WushError) as e:       # the tiled layout needs K % 64 == 0
        P.wush_quantize_f32_nvfp4(torch.zeros((4, 96), device="cuda"), one, G.empty_u8(32 * 48), G.empty_u8(32 * 6),
                                  layout=1)
    assert e.value.code == 2


def test_offsets_beyond_4_gib(P, G):
    """Buffers larger than 4 GiB (2^21 + 100 tokens of 4096 channels: X 17 GB, codes 4.3 GB; 1100 output
    channels: 4.6 GB of BF16): the quantizer and the GEMM give, for row ranges at the start, around the
    4 GiB marks of X, of the codes and of Y, and at the end, exactly the bytes the same rows give as a
    small batch (parity of small batches with the oracle is tested above).  A 32-bit offset anywhere in
    the path would send those rows elsewhere."""
    import torch
    P.wush_debug_set(P.WUSH_DEBUG_W4_SKINNY, 0)     # the small batches on the big batch's kernel: same accumulation order
    M, K, N = (1 << 21) + 100, 4096, 1100
    g = torch.Generator(device="cuda").manual_seed(21)
    X = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, M, 1 << 18):
        X[r0:r0 + (1 << 18)].normal_(generator=g)
    T = G.bf16_dev(I.make_transforms_random(K // 16, 6, block=16))
    W = (torch.randn((N, K), device="cuda", generator=g) * 0.05).to(torch.bfloat16)
    tsx, tsw = _f32_dev(0.01), torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = G.empty_u8(P.wush_prepare_weight_nvfp4_workspace(K))
    y_mark = (1 << 32) // (2 * N)
    ranges = [(0, 64), ((1 << 19) - 32, (1 << 19) + 32), (y_mark - 32, y_mark + 32), ((1 << 21) - 32, (1 << 21) + 32),
              (M - 70, M)]
    for layout in (0, 1):
        (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, layout), P.wush_packed_sizes_nvfp4(N, K, layout)
        assert xcb > (1 << 32)
        Xq, Xs, Wq, Ws = G.empty_u8(xcb), G.empty_u8(xsb), G.empty_u8(wcb), G.empty_u8(wsb)
        P.wush_prepare_weight_nvfp4(W, T, Wq, Ws, tsw, ws, layout=layout)
        P.wush_quantize_act_nvfp4(X, T, tsx, Xq, Xs, layout=layout)
        Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        P.wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Y, layout=layout, K=K)
        if layout:
            qu, su = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
            P.wush_unpack_tiled_nvfp4(Xq, Xs, M, K, qu, su)
        else:
            qu, su = Xq.view(M, K // 2), Xs.view(M, K // 16)
        torch.cuda.synchronize()
        assert not bool(Y[-4096:].isnan().any()) and not bool(Y[:4096].isnan().any())
        for lo, hi in ranges:
            m = hi - lo
            q, s_ = G.empty_u8(m, K // 2), G.empty_u8(m, K // 16)
            P.wush_quantize_act_nvfp4(X[lo:hi], T, tsx, q, s_)
            cb, sb = P.wush_packed_sizes_nvfp4(m, K, layout)
            ql, sl = G.empty_u8(cb), G.empty_u8(sb)
            P.wush_quantize_act_nvfp4(X[lo:hi], T, tsx, ql, sl, layout=layout)
            y = torch.full((m, N), float("nan"), dtype=torch.bfloat16, device="cuda")
            P.wush_linear_nvfp4(ql, sl, tsx, Wq, Ws, tsw, y, layout=layout, K=K)
            torch.cuda.synchronize()
            assert torch.equal(q, qu[lo:hi]) and torch.equal(s_, su[lo:hi]), (layout, lo, hi)
            assert torch.equal(y, Y[lo:hi]), (layout, lo, hi)
        del Xq, Xs, Y, qu, su
