"""GPU parity of the INT4 variant (32 x 32 transforms, two's-complement codes, BF16 scale
per 32 = Gaussian-MSE-optimal step times the group RMS) against oracle/wush_int4_oracle.py,
through the C ABI.  Bars: quantizer bit-exact when both sides see the same FP32 values;
transformed values within 1e-5 of the group AbsMax; codes against the all-FP64 path differ
only next to a decision boundary; GEMM relative Frobenius error <= 2e-3 (BF16 output) and
<= 1e-5 (FP32 output)."""
import numpy as np
import pytest

import wush_inputs as I
from oracle import wush_int4_oracle as Q
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
        _cache[name] = (cfg, L, X, W, O.round_to_bf16(O.build_transforms(W, Xc, 1e-2)))
    return _cache[name]


def _u16(t):
    """GPU u8 tensor [rows][2 * groups] -> numpy uint16 [rows][groups]."""
    return np.ascontiguousarray(t.cpu().numpy()).view(np.uint16)


def _adversarial_groups():
    rows = []
    for scale in (1.0, 3.7e-3, 911.0):
        s = np.float32(O.bf16_bits_to_f64(O.bf16_values_to_bits(O.round_to_bf16(np.array([scale]))))[0])
        for shift in (0.0, 1e-3):
            g = np.zeros(32, dtype=np.float32)
            halves = (np.arange(-9, 8) + 0.5).astype(np.float32)         # every rounding midpoint, and past both ends
            g[:17] = halves * s * np.float32(1 + shift)
            g[17:] = np.float32(0.3) * s
            rows.append(g)
    rows.append(np.zeros(32, dtype=np.float32))
    tiny = np.zeros(32, dtype=np.float32)
    tiny[3], tiny[9] = np.float32(1e-40), -np.float32(3e-39)              # scale below BF16's normal range
    rows.append(tiny)
    big = np.full(32, 1e30, dtype=np.float32)
    big[::3] *= -1
    rows.append(big)
    return np.stack(rows)


def test_quantizer_tap_bit_exact(P, G):
    import torch
    adv = _adversarial_groups()
    rnd = I.random_f32((257, 32 * 9), seed=21, spread=8.0)
    pad = (-adv.shape[0]) % 9
    adv = np.concatenate([adv, np.zeros((pad, 32), np.float32)]).reshape(-1, 32 * 9)
    Y = np.concatenate([rnd, adv]).astype(np.float32)
    M, K = Y.shape
    q, s = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_quantize_f32_int4(torch.from_numpy(Y).cuda(), q, s)
    torch.cuda.synchronize()
    # the kernel does exactly the steps it states (bit for bit) ...
    qr, sr = KM.int4_steps(Y, np.float32)
    assert np.array_equal(_u16(s), sr)
    assert np.array_equal(G.host(q), Q.pack_codes(qr))
    # ... and those steps differ from the definition (FP64, numpy's sum, a true division) only next to a
    # rounding boundary of the scale or of a code (values beyond FP32's square range aside: the last row)
    fin = np.isfinite(Y.astype(np.float64) ** 2).all(axis=1) & (np.abs(Y).max(axis=1) < 1e18)
    qd, sd = Q.quantize_int4(Y[fin])
    rate, unexplained = KM.int4_explained(Y[fin].astype(np.float64), qr[fin], sr[fin], qd, sd, tol=2e-6)
    assert unexplained == 0, (rate, unexplained)


@pytest.mark.parametrize("name", list(SHAPES))
def test_transform_quant(P, G, name):
    import torch
    cfg, L, X, W, T = _layer(name)
    M, K = cfg.M, cfg.K
    Xd, Td = G.bf16_dev(L["X"]), G.bf16_dev(O.bf16_values_to_bits(T))
    Xq, Xs = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    dbg = torch.full((M, K), float("nan"), dtype=torch.float32, device="cuda")
    P.wush_quantize_act_int4(Xd, Td, Xq, Xs, dbg_Yt=dbg)
    Xq2, Xs2 = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_quantize_act_int4(Xd, Td, Xq2, Xs2)
    torch.cuda.synchronize()
    xq, xs, yt = G.host(Xq), _u16(Xs), G.host(dbg)
    assert np.array_equal(xq, G.host(Xq2)) and np.array_equal(xs, _u16(Xs2))
    # (1) quantizer bit-exact on the kernel's own FP32 values
    assert np.isfinite(yt).all()
    qr, sr = KM.int4_steps(yt, np.float32)
    assert np.array_equal(xs, sr)
    assert np.array_equal(xq, Q.pack_codes(qr))
    # (2) transformed values against FP64
    Yt = O.transform_act(X, T)
    amax = np.max(np.abs(Yt.reshape(M, K // 32, 32)), axis=-1)
    err = np.max(np.abs(yt.astype(np.float64) - Yt).reshape(M, K // 32, 32), axis=-1)
    assert np.max(err / amax) <= 1e-5
    # (3) codes against the all-FP64 path
    q64, s64 = Q.quantize_int4(Yt)
    rate, unexplained = KM.int4_explained(Yt, Q.unpack_codes(xq), xs, q64, s64, tol=1e-5)
    assert rate <= 1e-3 and unexplained == 0, (rate, unexplained)


@pytest.mark.parametrize("name", list(SHAPES))
def test_prepare_weight(P, G, name):
    cfg, L, X, W, T = _layer(name)
    N, K = cfg.N, cfg.K
    Wd, Td = G.bf16_dev(L["W"]), G.bf16_dev(O.bf16_values_to_bits(T))
    Wq, Ws = G.empty_u8(N, K // 2), G.empty_u8(N, K // 16)
    ws = G.empty_u8(P.wush_prepare_weight_workspace(N, K))
    P.wush_prepare_weight_int4(Wd, Td, Wq, Ws, ws)
    P.wush_workspace_status(ws, K)
    Wt = O.transform_weight(W, T)
    qr, sr = Q.quantize_int4(Wt)
    rate, unexplained = KM.int4_explained(Wt, Q.unpack_codes(G.host(Wq)), _u16(Ws), qr, sr, tol=1e-9)
    assert rate <= 1e-3 and unexplained == 0, (rate, unexplained)


def test_prepare_weight_flags_singular_block(P, G):
    K, N = 64, 40
    T = np.stack([np.eye(32), np.eye(32)])
    T[1, 5, :] = 0.0
    Wd = G.bf16_dev(I.f32_to_bf16_bits(I.random_f32((N, K), 5, 1.0)))
    Wq, Ws = G.empty_u8(N, K // 2), G.empty_u8(N, K // 16)
    ws = G.empty_u8(P.wush_prepare_weight_workspace(N, K))
    P.wush_prepare_weight_int4(Wd, G.bf16_dev(O.bf16_values_to_bits(T)), Wq, Ws, ws)
    with pytest.raises(P.WushError) as e:
        P.wush_workspace_status(ws, K)
    assert e.value.code == 7


def _random_operand(rng, rows, K, lo_exp, hi_exp):
    q = rng.integers(-8, 8, (rows, K)).astype(np.int8)
    s = O.round_to_bf16(np.exp2(rng.uniform(lo_exp, hi_exp, (rows, K // 32))) * rng.uniform(1, 2, (rows, K // 32)))
    return q, O.bf16_values_to_bits(s)


GEMM_SHAPES = [(16, 256, 64), (77, 45, 128), (300, 520, 192), (257, 256, 1024), (512, 768, 4096), (1, 32, 256)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_linear_against_oracle(P, G, M, N, K, out):
    """GEMM alone: both sides start from the same codes and BF16 scales (spread over FP16's normal range)."""
    import torch
    rng = np.random.default_rng(2000 + M + N + K)
    xq, xs = _random_operand(rng, M, K, -13, 9)
    wq, ws_ = _random_operand(rng, N, K, -10, -2)
    ref = Q.linear_dequant(xq, xs, wq, ws_)
    f32 = out == "f32"
    Y = torch.full((M, N + 8), float("nan"), dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")
    P.wush_linear_int4(G.u8_dev(Q.pack_codes(xq)), G.u8_dev(xs.view(np.uint8)), G.u8_dev(Q.pack_codes(wq)),
                       G.u8_dev(ws_.view(np.uint8)), Y[:, :N], out_dtype=1 if f32 else 0)
    torch.cuda.synchronize()
    y = Y.float().cpu().numpy().astype(np.float64)
    assert np.isnan(y[:, N:]).all()
    assert O.rel_fro(y[:, :N], ref) <= (1e-5 if f32 else 2e-3)


def _tile_operand(packed, scale_bytes):
    """Canonical packed codes [rows][K/2] and scale bytes [rows][K/16] (two BF16 numbers per 64-element K
    step) -> the tiled buffers, from the statement of the layout: rows padded to 32; the 16-byte chunk
    (row, kt, hh) at ((((row / 32) KT + kt) 2 + hh) 32 + row % 32) 16, the scale dword (row, kt) at
    (((row / 32) KT + kt) 32 + row % 32) 4."""
    rows, K = packed.shape[0], packed.shape[1] * 2
    KT, RB = K // 64, (rows + 31) // 32
    pq = np.zeros((RB * 32, KT, 2, 16), dtype=np.uint8)
    pq[:rows] = packed.reshape(rows, KT, 2, 16)
    ps = np.zeros((RB * 32, KT, 4), dtype=np.uint8)
    ps[:rows] = scale_bytes.reshape(rows, KT, 4)
    q = pq.reshape(RB, 32, KT, 2, 16).transpose(0, 2, 3, 1, 4)
    sc = ps.reshape(RB, 32, KT, 4).transpose(0, 2, 1, 3)
    return np.ascontiguousarray(q).reshape(-1), np.ascontiguousarray(sc).reshape(-1)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("K", [320, 384])
@pytest.mark.parametrize("width", ["2", "3", "4"])
def test_linear_every_tile_width(P, G, width, K, layout):
    """The three tile widths on a shape with several tiles and ragged edges in both directions, GEMM alone.
    An odd number of 64-element K steps (K = 320) takes the kernel that stages both operands in LDS, an
    even one (K = 384) the one that converts W in registers; both read either layout."""
    import torch
    _force_width(P, width)
    M, N = 300, 700
    rng = np.random.default_rng(91 + K)
    xq, xs = _random_operand(rng, M, K, -13, 9)
    wq, ws_ = _random_operand(rng, N, K, -10, -2)
    ref = Q.linear_dequant(xq, xs, wq, ws_)
    xp, wp = Q.pack_codes(xq), Q.pack_codes(wq)
    xsb, wsb = xs.view(np.uint8).reshape(M, -1), ws_.view(np.uint8).reshape(N, -1)
    if layout:
        (xp, xsb), (wp, wsb) = _tile_operand(xp, xsb), _tile_operand(wp, wsb)
    Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    P.wush_linear_int4(G.u8_dev(xp), G.u8_dev(xsb), G.u8_dev(wp), G.u8_dev(wsb), Y, layout=layout, out_dtype=1, K=K)
    torch.cuda.synchronize()
    assert O.rel_fro(Y.cpu().numpy().astype(np.float64), ref) <= 1e-5


@pytest.mark.parametrize("kernel", [1, 2, 0, -1], ids=["streaming_split_k", "streaming_shared_x", "tiled", "library_choice"])
@pytest.mark.parametrize("M", [1, 2, 7, 16, 31, 32, 33, 48, 64, 65, 100, 128])
@pytest.mark.parametrize("K", [64, 320, 1024])
def test_linear_few_tokens_on_either_kernel(P, G, K, M, kernel):
    """Up to 128 tokens the tiled layout takes a weight-streaming kernel (one workgroup per 32 output
    channels, K split over its four waves; beyond 64 tokens also one workgroup per 128 output channels whose
    waves share the converted activations through LDS); they and the tiled kernel are forced in turn on a ragged
    shape, FP32 and BF16 output, against the oracle on the same codes and BF16 scales."""
    import torch
    N = 1000
    rng = np.random.default_rng(5000 + 7 * M + K)
    xq, xs = _random_operand(rng, M, K, -13, 9)
    wq, ws_ = _random_operand(rng, N, K, -10, -2)
    ref = Q.linear_dequant(xq, xs, wq, ws_)
    (xp, xsb), (wp, wsb) = (_tile_operand(Q.pack_codes(xq), xs.view(np.uint8).reshape(M, -1)),
                            _tile_operand(Q.pack_codes(wq), ws_.view(np.uint8).reshape(N, -1)))
    P.wush_debug_set(P.WUSH_DEBUG_W4_SKINNY, kernel)
    for f32 in (True, False):
        Y = torch.full((M, N + 8), float("nan"), dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")
        P.wush_linear_int4(G.u8_dev(xp), G.u8_dev(xsb), G.u8_dev(wp), G.u8_dev(wsb), Y[:, :N], layout=1,
                           out_dtype=1 if f32 else 0, K=K)
        torch.cuda.synchronize()
        y = Y.float().cpu().numpy().astype(np.float64)
        assert np.isnan(y[:, N:]).all()
        assert np.isfinite(y[:, :N]).all()
        assert O.rel_fro(y[:, :N], ref) <= (1e-5 if f32 else 2e-3), (f32, O.rel_fro(y[:, :N], ref))


@pytest.mark.parametrize("width", ["2", "3", "4"])
def test_layer_end_to_end_both_layouts(P, G, width):
    import torch
    _force_width(P, width)
    cfg, L, X, W, T = _layer("tiles")
    M, N, K = cfg.M, cfg.N, cfg.K
    Xd, Wd, Td = G.bf16_dev(L["X"]), G.bf16_dev(L["W"]), G.bf16_dev(O.bf16_values_to_bits(T))
    ws = G.empty_u8(P.wush_prepare_weight_workspace(N, K))
    outs = []
    for lay in (0, 1):
        (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, lay), P.wush_packed_sizes_nvfp4(N, K, lay)
        Xq, Xs, Wq, Ws = G.empty_u8(xcb), G.empty_u8(xsb), G.empty_u8(wcb), G.empty_u8(wsb)
        P.wush_prepare_weight_int4(Wd, Td, Wq, Ws, ws, layout=lay)
        P.wush_quantize_act_int4(Xd, Td, Xq, Xs, layout=lay)
        Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        P.wush_linear_int4(Xq, Xs, Wq, Ws, Y, layout=lay, out_dtype=1, K=K)
        if lay:   # the tiled buffers are a permutation of the canonical ones
            qu, su = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
            P.wush_unpack_tiled_nvfp4(Xq, Xs, M, K, qu, su)
            torch.cuda.synchronize()
            assert torch.equal(qu, outs[0][1].view(M, K // 2)) and torch.equal(su, outs[0][2].view(M, K // 16))
        outs.append((Y, Xq, Xs))
    torch.cuda.synchronize()
    assert torch.equal(outs[0][0], outs[1][0])
    ref = Q.layer_forward(X, W, T)
    y = outs[1][0].cpu().numpy().astype(np.float64)
    assert O.rel_fro(y, ref) <= 2e-3
    exact = X @ W.T
    assert abs(O.rel_fro(y, exact) - O.rel_fro(ref, exact)) <= 1e-3


def test_transform_quant_is_independent_of_the_launch_shape(P, G):
    """A large, ragged batch (workgroups of two wave groups, nine tiles each, a last tile of three tokens)
    gives, row for row, the bytes the same rows give in small batches, in both layouts."""
    import torch
    M, K = 4099, 8192
    X = torch.from_numpy(I.random_f32((M, K), seed=43, spread=2.0)).cuda().to(torch.bfloat16)
    T = G.bf16_dev(I.make_transforms_random(K // 32, 5))
    Xq, Xs = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_quantize_act_int4(X, T, Xq, Xs)
    cb, sb = P.wush_packed_sizes_nvfp4(M, K, 1)
    Xqt, Xst = G.empty_u8(cb), G.empty_u8(sb)
    P.wush_quantize_act_int4(X, T, Xqt, Xst, layout=1)
    Xqu, Xsu = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16)
    P.wush_unpack_tiled_nvfp4(Xqt, Xst, M, K, Xqu, Xsu)
    torch.cuda.synchronize()
    assert torch.equal(Xqu, Xq) and torch.equal(Xsu, Xs)
    for lo, hi in ((0, 256), (1500, 1533), (4064, 4099)):
        q, s_ = G.empty_u8(hi - lo, K // 2), G.empty_u8(hi - lo, K // 16)
        P.wush_quantize_act_int4(X[lo:hi], T, q, s_)
        torch.cuda.synchronize()
        assert torch.equal(q, Xq[lo:hi]) and torch.equal(s_, Xs[lo:hi]), (lo, hi)


@pytest.mark.parametrize("name", ["c2", "c5"])
def test_bench_shapes_full_size(P, G, name):
    """The configurations bench.py times for the workloads i2 (2048 x 4096 -> 6144) and i5 (8192 x 8192 ->
    57344), tiled layout, BF16 output: sampled token rows, weight rows and output entries against the oracle."""
    import torch
    L = I.make_layer(I.CONFIGS[name])
    cfg = L["cfg"]
    M, K, N = cfg.M, cfg.K, cfg.N
    T = np.empty((K // 32, 32, 32))
    for b in range(K // 32):
        sl = slice(32 * b, 32 * b + 32)
        T[b] = O.wush_block(O.second_moment(O.bf16_bits_to_f64(L["W"][:, sl])),
                            O.second_moment(O.bf16_bits_to_f64(L["X_cal"][:, sl])), 1e-2)
    T = O.round_to_bf16(T)
    rng = np.random.default_rng(23)
    rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, 48)]))
    cols = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, 256)]))
    Xd, Wd, Td = G.bf16_dev(L["X"]), G.bf16_dev(L["W"]), G.bf16_dev(O.bf16_values_to_bits(T))
    (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, 1), P.wush_packed_sizes_nvfp4(N, K, 1)
    Xq, Xs, Wq, Ws = G.empty_u8(xcb), G.empty_u8(xsb), G.empty_u8(wcb), G.empty_u8(wsb)
    ws = G.empty_u8(P.wush_prepare_weight_workspace(N, K))
    P.wush_prepare_weight_int4(Wd, Td, Wq, Ws, ws, layout=1)
    P.wush_workspace_status(ws, K)
    P.wush_quantize_act_int4(Xd, Td, Xq, Xs, layout=1)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.wush_linear_int4(Xq, Xs, Wq, Ws, Y, layout=1, K=K)
    Xqc, Xsc, Wqc, Wsc = G.empty_u8(M, K // 2), G.empty_u8(M, K // 16), G.empty_u8(N, K // 2), G.empty_u8(N, K // 16)
    P.wush_unpack_tiled_nvfp4(Xq, Xs, M, K, Xqc, Xsc)
    P.wush_unpack_tiled_nvfp4(Wq, Ws, N, K, Wqc, Wsc)
    torch.cuda.synchronize()
    assert not bool(Y.isnan().any())
    X = O.bf16_bits_to_f64(L["X"][rows])
    Yt = O.transform_act(X, T)
    xq, xs = Q.unpack_codes(Xqc[rows.tolist()].cpu().numpy()), _u16(Xsc[rows.tolist()])
    q64, s64 = Q.quantize_int4(Yt)
    rate, unexplained = KM.int4_explained(Yt, xq, xs, q64, s64, tol=1e-5)
    assert rate <= 1e-3 and unexplained == 0, ("activation codes", rate, unexplained)
    Wt = O.transform_weight(O.bf16_bits_to_f64(L["W"][cols]), T)
    qw, sw = Q.quantize_int4(Wt)
    wq, wsc = Q.unpack_codes(Wqc[cols.tolist()].cpu().numpy()), _u16(Wsc[cols.tolist()])
    rate, unexplained = KM.int4_explained(Wt, wq, wsc, qw, sw, tol=1e-9)
    assert rate <= 1e-3 and unexplained == 0, ("weight codes", rate, unexplained)
    y = O.bf16_bits_to_f64(G.host(Y[rows.tolist()][:, cols.tolist()].contiguous()))
    own = Q.linear_dequant(xq, xs, wq, wsc)
    assert O.rel_fro(y, own) <= 2e-3
    ref = Q.linear_dequant(q64, s64, qw, sw)
    exact = X @ O.bf16_bits_to_f64(L["W"][cols]).T
    q_err = O.rel_fro(ref, exact)
    assert O.rel_fro(y, ref) <= max(2e-3, 0.05 * q_err) and q_err < 0.25, (O.rel_fro(y, ref), q_err)
    # every output tile: FP32 output, one seeded token row per band of 128 rows (the kernel's tiles are 256 rows
    # high) x ALL N columns against the dequantized FP64 product of the GPU's own codes (exact inputs: FP32
    # accumulation is the only difference), and BF16 == RNE(FP32) bit for bit
    Y32 = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    P.wush_linear_int4(Xq, Xs, Wq, Ws, Y32, layout=1, out_dtype=1, K=K)
    torch.cuda.synchronize()
    assert not bool(Y32.isnan().any())
    band = np.array([min(b + int(rng.integers(0, 128)), M - 1) for b in range(0, M, 128)])
    y32 = Y32[band.tolist()].cpu().numpy()
    del Y32
    assert np.array_equal(G.host(Y[band.tolist()].contiguous()), O.bf16_values_to_bits(O.round_to_bf16(y32.astype(np.float64))))
    xq_b, xs_b = Q.unpack_codes(Xqc[band.tolist()].cpu().numpy()), _u16(Xsc[band.tolist()])
    xn = np.linalg.norm(Q.dequantize_int4(xq_b, xs_b), axis=1)
    wq_host, ws_host = Wqc.cpu().numpy(), _u16(Wsc)

    def chunk(c0, width=2048):
        c1 = min(N, c0 + width)
        wc = Q.unpack_codes(wq_host[c0:c1])
        part = Q.linear_dequant(xq_b, xs_b, wc, ws_host[c0:c1])
        d = y32[:, c0:c1].astype(np.float64) - part
        wn = np.linalg.norm(Q.dequantize_int4(wc, ws_host[c0:c1]), axis=1)
        return float(np.sum(d * d)), float(np.sum(part * part)), float(np.max(np.abs(d) / (xn[:, None] * wn[None, :] + 1e-300)))

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=8) as ex:
        parts = list(ex.map(chunk, range(0, N, 2048)))
    num, den, worst = sum(q[0] for q in parts), sum(q[1] for q in parts), max(q[2] for q in parts)
    print(f"int4 {name}: every-tile check on {len(band)} rows x {N} columns: rel. Frobenius {np.sqrt(num / den):.2e}, "
          f"largest element error / (|x| |w|) {worst:.2e}")
    assert np.sqrt(num / den) <= 1e-5 and worst <= 1e-5
    # the same weights through the kernels for few tokens (16: K split over the waves, the shape bench.py times as
    # di2 / di5; 100: activations shared through LDS on the wide layer), every output element, FP32 output
    for m in (16, 100):
        (mcb, msb) = P.wush_packed_sizes_nvfp4(m, K, 1)
        xq_m, xs_m = G.empty_u8(mcb), G.empty_u8(msb)
        P.wush_quantize_act_int4(Xd[:m], Td, xq_m, xs_m, layout=1)
        Ym = torch.full((m, N), float("nan"), dtype=torch.float32, device="cuda")
        P.wush_linear_int4(xq_m, xs_m, Wq, Ws, Ym, layout=1, out_dtype=1, K=K)
        torch.cuda.synchronize()
        y32 = Ym.cpu().numpy()
        assert np.isfinite(y32).all()
        xq_b, xs_b = Q.unpack_codes(Xqc[:m].cpu().numpy()), _u16(Xsc[:m])             # rows of a batch do not depend on its size
        xn = np.linalg.norm(Q.dequantize_int4(xq_b, xs_b), axis=1)
        with ThreadPoolExecutor(max_workers=8) as ex:
            parts = list(ex.map(chunk, range(0, N, 2048)))
        num, den, worst = sum(q[0] for q in parts), sum(q[1] for q in parts), max(q[2] for q in parts)
        print(f"int4 {name}, {m} tokens: rel. Frobenius {np.sqrt(num / den):.2e}, largest element error / (|x| |w|) {worst:.2e}")
        assert np.sqrt(num / den) <= 1e-5 and worst <= 1e-5


def test_argument_validation(P, G):
    import torch
    Y = torch.empty((4, 4), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(P.WushError) as e:        # K = 96 is not a multiple of 64
        P.wush_linear_int4(G.empty_u8(4, 48), G.empty_u8(4, 6), G.empty_u8(4, 48), G.empty_u8(4, 6), Y)
    assert e.value.code == 2
    with pytest.raises(P.WushError) as e:
        P.wush_linear_int4(G.empty_u8(4, 64), None, G.empty_u8(4, 64), G.empty_u8(4, 8), Y)
    assert e.value.code == 1
    with pytest.raises(P.WushError) as e:        # unknown layout
        P.wush_quantize_f32_int4(torch.zeros((4, 64), device="cuda"), G.empty_u8(4, 32), G.empty_u8(4, 4), layout=7)
    assert e.value.code == 4


def test_offsets_beyond_4_gib(P, G):
    """Buffers larger than 4 GiB (2^21 + 100 tokens of 4096 channels: X 17 GB, codes 4.3 GB; 1100 output
    channels: 4.6 GB of BF16): the quantizer and the GEMM give, for row ranges at the start, around the
    4 GiB marks of X, of the codes and of Y, and at the end, exactly the bytes the same rows give as a
    small batch (parity of small batches with the oracle is tested above).  A 32-bit offset anywhere in
    the path would send those rows elsewhere."""
    import torch
    P.wush_debug_set(P.WUSH_DEBUG_W4_SKINNY, 0)     # the small batches on the big batch's kernel: same accumulation order
    M, K, N = (1 << 21) + 100, 4096, 1100
    g = torch.Generator(device="cuda").manual_seed(31)
    X = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, M, 1 << 18):
        X[r0:r0 + (1 << 18)].normal_(generator=g)
    T = G.bf16_dev(I.make_transforms_random(K // 32, 7))
    W = (torch.randn((N, K), device="cuda", generator=g) * 0.05).to(torch.bfloat16)
    ws = G.empty_u8(P.wush_prepare_weight_workspace(N, K))
    y_mark = (1 << 32) // (2 * N)
    ranges = [(0, 64), ((1 << 19) - 32, (1 << 19) + 32), (y_mark - 32, y_mark + 32), ((1 << 21) - 32, (1 << 21) + 32),
              (M - 70, M)]
    for layout in (0, 1):
        (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, layout), P.wush_packed_sizes_nvfp4(N, K, layout)
        assert xcb > (1 << 32)
        Xq, Xs, Wq, Ws = G.empty_u8(xcb), G.empty_u8(xsb), G.empty_u8(wcb), G.empty_u8(wsb)
        P.wush_prepare_weight_int4(W, T, Wq, Ws, ws, layout=layout)
        P.wush_quantize_act_int4(X, T, Xq, Xs, layout=layout)
        Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        P.wush_linear_int4(Xq, Xs, Wq, Ws, Y, layout=layout, K=K)
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
            P.wush_quantize_act_int4(X[lo:hi], T, q, s_)
            cb, sb = P.wush_packed_sizes_nvfp4(m, K, layout)
            ql, sl = G.empty_u8(cb), G.empty_u8(sb)
            P.wush_quantize_act_int4(X[lo:hi], T, ql, sl, layout=layout)
            y = torch.full((m, N), float("nan"), dtype=torch.bfloat16, device="cuda")
            P.wush_linear_int4(ql, sl, Wq, Ws, y, layout=layout, K=K)
            torch.cuda.synchronize()
            assert torch.equal(q, qu[lo:hi]) and torch.equal(s_, su[lo:hi]), (layout, lo, hi)
            assert torch.equal(y, Y[lo:hi]), (layout, lo, hi)
        del Xq, Xs, Y, qu, su
