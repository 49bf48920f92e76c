"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: quantized codes, scales and int32 accumulators bit-exact; fp16 outputs within 1e-3 of the
oracle's fp64 result, as max-abs error normalised by the largest reference magnitude.
"""
import numpy as np
import pytest

import oracle
from paper_2512_23367_amd import binding as ql
from paper_2512_23367_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-3


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


@pytest.fixture(autouse=True)
def _auto_variant():
    yield
    ql.ql_set_kernel_variant(0)


# ------------------------------------------------------------------ quantizers
@pytest.mark.parametrize("M,K,ldx", [(64, 512, None), (33, 1536, None), (5, 11008, None), (3, 64, None),
                                     (7, 4096, 4104), (1, 4096, None), (2, 6144, None), (4, 40960, None),
                                     (513, 512, None), (600, 1536, 1544), (515, 16384, None), (40, 40960, None)])
def test_act_quant_bit_exact(G, M, K, ldx):
    x = synth.activations(M, K, 0, "single")
    x[M // 2, :] *= np.float16(0.01) if M > 1 else np.float16(1)
    xq_o, sx_o = oracle.quant_act_per_token(x)
    xq_g, sx_g, xk = G.gpu_quant_act(x, ldx)
    assert (xq_g == xq_o).all()
    assert (sx_g.view(np.uint32) == sx_o.view(np.uint32)).all()
    # the kernel-layout copy holds the same codes: it must equal the repack of the oracle's codes on valid rows
    a = xk.cpu().numpy().view(np.int8)
    b = G.repack_act(xq_o).cpu().numpy().view(np.int8)
    rows_valid = _kernel_layout_mask(M, K)
    assert (a[rows_valid] == b[rows_valid]).all()


def _kernel_layout_mask(M, K):
    """Boolean mask over the kernel-layout bytes that belong to rows < M (tile order: 32 rows x 32 k per 1 KiB,
    lane = row%32 + 32*((k%32)//16), 16 bytes per lane)."""
    Mp = (M + 31) // 32 * 32
    idx = np.arange(Mp * K)
    tile, within = idx // 1024, idx % 1024
    lane = within // 16
    row = (tile // (K // 32)) * 32 + lane % 32
    return row < M


def test_act_quant_zero_rows_and_ties(G):
    x = np.zeros((4, 64), dtype=np.float16)
    x[1, :7] = [127.0, 63.5, -62.5, 0.5, -1.5, 2.5, 0.0]       # inv = 1: every .5 is a tie
    x[2, :4] = [1.0, -0.5, 0.25, 2.0]
    xq_o, sx_o = oracle.quant_act_per_token(x)
    xq_g, sx_g, _ = G.gpu_quant_act(x)
    assert xq_g[1, :7].tolist() == [127, 64, -62, 0, -2, 2, 0]
    assert (xq_g == xq_o).all() and (sx_g == sx_o).all()
    assert sx_g[0] == 1 and sx_g[3] == 1 and (xq_g[0] == 0).all()


@pytest.mark.parametrize("N,K", [(512, 512), (100, 1536), (33, 4096)])
def test_weight_quant_int8_bit_exact_and_export(G, N, K):
    w = synth.weights(N, K, 0, "single")
    w[1] = 0
    wq_o, sw_o = oracle.quant_weight_int8(w)
    g = G.gpu_quant_weight(w, 8, 0)
    assert (g["canon"] == wq_o).all()
    assert (g["scales"].view(np.uint32) == sw_o.view(np.uint32)).all()
    back, _ = G.gpu_export(g["kernel"], N, K, 8, 0)
    assert (back == wq_o).all()


@pytest.mark.parametrize("N,K", [(512, 512), (100, 1536), (33, 4096)])
def test_weight_quant_int4_bit_exact_and_export(G, N, K):
    w = synth.weights(N, K, 0, "single")
    w[1, :128] = 0
    w[2, 128:256] *= np.float16(1e-4)
    packed_o, _, s_o = oracle.quant_weight_int4(w, 128)
    g = G.gpu_quant_weight(w, 4, 128)
    assert (g["canon"] == packed_o).all()
    assert (g["scales"].view(np.uint16) == s_o.view(np.uint16)).all()
    back, sback = G.gpu_export(g["kernel"], N, K, 4, 128)
    assert (back == packed_o).all() and (sback.view(np.uint16) == s_o.view(np.uint16)).all()


# --------------------------------------------------------------- accumulators
PREFILL_VARIANTS = [4, 6, 11, 13, 15, 17, 19, 20, 23, 26, 35, 37, 39, 43]   # 26..43: 16x16x64 matrix instruction
SHAPES_ACC = [(64, 512, 512), (100, 192, 200), (300, 1024, 520), (257, 256, 33)]


@pytest.mark.parametrize("variant", PREFILL_VARIANTS)
@pytest.mark.parametrize("M,K,N", SHAPES_ACC)
def test_w8a8_accumulators_bit_exact_prefill(G, variant, M, K, N):
    if variant in (19, 39) and K % 128:
        pytest.skip("this variant stages 128 k at a time (the library falls back to a 64-k variant)")
    rng = np.random.default_rng(M + K + N)
    xq = rng.integers(-127, 128, (M, K), dtype=np.int8)
    w = synth.weights(N, K, 0, "single")
    g = G.gpu_quant_weight(w, 8, 0)
    ql.ql_set_kernel_variant(variant)
    acc, _ = G.gpu_acc(xq, g)
    assert (acc == oracle.igemm(xq, g["canon"])).all()


@pytest.mark.parametrize("M", [1, 8, 16, 17, 32])
@pytest.mark.parametrize("K,N", [(512, 512), (4096, 200), (11008, 48), (192, 33)])
def test_w8a8_accumulators_bit_exact_decode(G, M, K, N):
    rng = np.random.default_rng(M + K + N)
    xq = rng.integers(-127, 128, (M, K), dtype=np.int8)
    g = G.gpu_quant_weight(synth.weights(N, K, 0, "single"), 8, 0)
    acc, _ = G.gpu_acc(xq, g)
    assert (acc == oracle.igemm(xq, g["canon"])).all()


DECODE_VARIANTS = [101, 102, 103, 104, 106, 108, 111, 121]   # 1..8 channel groups per workgroup, 16 wavefronts, tokens from L2


@pytest.mark.parametrize("variant", DECODE_VARIANTS)
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,K,N", [(1, 1024, 200), (8, 4096, 136), (17, 512, 72), (32, 1536, 200), (33, 512, 72),
                                   (50, 1536, 200), (64, 4096, 136), (130, 1024, 200)])
def test_decode_variants_bit_exact_and_within_tolerance(G, variant, bits, M, K, N):
    rng = np.random.default_rng(M + K + N + bits)
    xq = rng.integers(-127, 128, (M, K), dtype=np.int8)
    w = synth.weights(N, K, 0, "single")
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    ql.ql_set_kernel_variant(variant)
    if bits == 8:
        acc, _ = G.gpu_acc(xq, g)
        assert (acc == oracle.igemm(xq, g["canon"])).all()
    else:
        _, total, part = oracle.igemm_grouped(xq, oracle.unpack_int4(g["canon"]), g["scales"], 128, want_partials=True)
        acc, gpart = G.gpu_acc(xq, g, want_partials=True)
        assert (acc == total).all() and (gpart == part).all()
    x = synth.activations(M, K, 0, "single")
    b = synth.bias(N, 0, "single")
    ref = (oracle.linear_w8a8(x, g["canon"], g["scales"], b) if bits == 8
           else oracle.linear_w4a8(x, g["canon"], g["scales"], 128, b))
    assert G.norm_err(G.gpu_linear(x, g, b), ref["y64"]) <= TOL


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M", [2, 40])
def test_largest_k_decode_and_prefill(G, bits, M):
    """K = 131072, the largest the interface accepts (no int32 accumulator can overflow below 133144)."""
    K, N = 131072, 40
    rng = np.random.default_rng(K + M + bits)
    xq = rng.integers(-127, 128, (M, K), dtype=np.int8)
    xq[0] = 127                                            # one token at the extreme
    w = synth.weights(N, K, 0, "single")
    w[1] = np.abs(w[1]).max()                              # one channel whose codes are all +127 / +7
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    if bits == 8:
        acc, _ = G.gpu_acc(xq, g)
        ref = oracle.igemm(xq, g["canon"])
        assert int(ref[0, 1]) == 127 * 127 * K             # the largest accumulator value there is
        assert (acc == ref).all()
    else:
        _, total, _ = oracle.igemm_grouped(xq, oracle.unpack_int4(g["canon"]), g["scales"], 128)
        acc, _ = G.gpu_acc(xq, g)
        assert (acc == total).all()


# ------------------------------------------------------------------ split-K (few tokens, long K)
@pytest.mark.parametrize("variant", [202, 203, 208, 302, 305])
@pytest.mark.parametrize("M,K,N", [(64, 4096, 200), (100, 1536, 264), (300, 2048, 520), (33, 11008, 48)])
def test_w8a8_split_k_accumulators_bit_exact(G, variant, M, K, N):
    """K split over several workgroups per tile + second kernel adding the int32 partial sums: still exact."""
    splits, T = variant % 100, 128 if variant < 300 else 256
    if K // 64 // splits < 1:
        pytest.skip("more splits than 64-k stages")
    rng = np.random.default_rng(M + K + N)
    xq = rng.integers(-127, 128, (M, K), dtype=np.int8)
    g = G.gpu_quant_weight(synth.weights(N, K, 0, "single"), 8, 0)
    ws = G.empty_bytes(splits * -(-M // T) * -(-N // T) * T * T * 4)
    ql.ql_set_kernel_variant(variant)
    acc, _ = G.gpu_acc(xq, g, ws=ws)
    assert (acc == oracle.igemm(xq, g["canon"])).all()
    with pytest.raises(ql.QlError):                        # the same call without the scratch it needs
        G.gpu_acc(xq, g)


@pytest.mark.parametrize("variant", [100, 101, 104, 108, 122, 123])   # automatic; 1/4/8 channel groups; blocks of 32/64 tokens
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,K,N,bias", [(33, 512, 96, False), (64, 4096, 200, True), (65, 1024, 136, True), (100, 1536, 1000, False),
                                        (128, 128, 33, True), (300, 2048, 520, False), (1024, 512, 72, True)])
def test_decode_kernels_on_blocks_of_64_tokens(G, variant, bits, M, K, N, bias):
    """From 33 tokens on the decode kernels work on blocks of 64 or 32 tokens (one grid row each, up to 1024 tokens): exact
    integer sums (int4: group partials too, for a row window that straddles blocks), fp16 output within tolerance
    and, for int8, equal to the tile kernels' up to the rounding of the last step."""
    x = synth.activations(M, K, 0, "single")
    w = synth.weights(N, K, 0, "single")
    b = synth.bias(N, 0, "single") if bias else None
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    xq, _ = oracle.quant_act_per_token(x)
    ql.ql_set_kernel_variant(variant)
    if bits == 8:
        ref = oracle.linear_w8a8(x, g["canon"], g["scales"], b)
        acc, _ = G.gpu_acc(xq, g)
        assert (acc == ref["acc"]).all()
    else:
        ref = oracle.linear_w4a8(x, g["canon"], g["scales"], 128, b)
        _, total, part = oracle.igemm_grouped(xq, oracle.unpack_int4(g["canon"]), g["scales"], 128, want_partials=True)
        row0 = max(0, min(M - 8, 60))
        acc, gpart = G.gpu_acc(xq, g, want_partials=True, row0=row0, nrows=min(8, M))
        assert (acc == total).all() and (gpart == part[row0:row0 + min(8, M)]).all()
    y = G.gpu_linear(x, g, b)
    assert G.norm_err(y, ref["y64"]) <= TOL
    ql.ql_set_kernel_variant(1)
    y1 = G.gpu_linear(x, g, b, extra_ws=32 << 20)
    ql.ql_set_kernel_variant(0)
    if bits == 8:
        # same integer sums; the fused epilogues may round the dequantized value differently in its last fp32 bit
        diff = y.view(np.uint16) != y1.view(np.uint16)
        assert diff.mean() < 1e-3
        assert np.abs(y.astype(np.float64) - y1.astype(np.float64))[diff].max(initial=0) <= \
            np.spacing(np.abs(y1[diff]).astype(np.float16)).astype(np.float64).max(initial=0)
    else:
        assert G.norm_err(y, y1.astype(np.float64)) <= 2e-3


def test_decode_kernels_refuse_more_than_1024_tokens(G):
    g = G.gpu_quant_weight(synth.weights(40, 128, 0, "single"), 8, 0)
    ql.ql_set_kernel_variant(100)
    try:
        with pytest.raises(ql.QlError):
            G.gpu_acc(np.zeros((1025, 128), dtype=np.int8), g)
    finally:
        ql.ql_set_kernel_variant(0)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,K,N,variant", [(64, 4096, 200, 204), (100, 1536, 264, 203), (200, 11008, 136, 1),
                                           (48, 4096, 520, 1), (300, 2048, 520, 302)])
def test_split_k_linear_within_tolerance_and_deterministic(G, bits, M, K, N, variant):
    x = synth.activations(M, K, 0, "single")
    w = synth.weights(N, K, 0, "single")
    b = synth.bias(N, 0, "single")
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    ref = (oracle.linear_w8a8(x, g["canon"], g["scales"], b) if bits == 8
           else oracle.linear_w4a8(x, g["canon"], g["scales"], 128, b))
    if bits == 4 and variant >= 300:
        variant = 203                                      # the int4 kernel has one tile shape
    ql.ql_set_kernel_variant(variant)
    y1 = G.gpu_linear(x, g, b, extra_ws=64 << 20)
    y2 = G.gpu_linear(x, g, b, extra_ws=64 << 20)
    assert np.isfinite(y1).all()
    assert G.norm_err(y1, ref["y64"]) <= TOL
    assert (y1.view(np.uint16) == y2.view(np.uint16)).all()
    # and the unsplit kernels agree to rounding (int8: same integer sums -- tested above -- so at most the last
    # fp32 bit of the dequantized value differs, which moves an fp16 result across a rounding boundary rarely)
    ql.ql_set_kernel_variant(13 if bits == 8 else 6)   # int4: any unsplit value selects its one tile kernel
    y0 = G.gpu_linear(x, g, b)
    if bits == 8:
        diff = y1.view(np.uint16) != y0.view(np.uint16)
        assert diff.mean() < 1e-3
        assert np.abs(y1.astype(np.float64) - y0.astype(np.float64))[diff].max(initial=0) <= \
            np.spacing(np.abs(y0[diff]).astype(np.float16)).astype(np.float64).max(initial=0)
    else:
        assert G.norm_err(y1, y0.astype(np.float64)) <= 2e-3


def test_w8a8_accumulator_extremes(G):
    K = 11008
    xq = np.full((2, K), 127, dtype=np.int8)
    xq[1] = -127
    w = np.ones((40, K), dtype=np.float16)
    w[1::2] = -1
    g = G.gpu_quant_weight(w, 8, 0)
    assert (np.abs(g["canon"]) == 127).all()
    acc, _ = G.gpu_acc(xq, g)
    assert (acc == oracle.igemm(xq, g["canon"])).all() and abs(int(acc[0, 0])) == 177548032
    ql.ql_set_kernel_variant(6)                            # the same through a prefill tile kernel
    acc, _ = G.gpu_acc(xq, g)
    assert (acc == oracle.igemm(xq, g["canon"])).all()


@pytest.mark.parametrize("M,K,N", [(64, 512, 512), (100, 256, 200), (300, 1024, 264), (1, 512, 512), (8, 4096, 200),
                                   (17, 1024, 48), (32, 11008, 64)])
def test_w4a8_accumulators_and_partials_bit_exact(G, M, K, N):
    rng = np.random.default_rng(M + K + N)
    xq = rng.integers(-127, 128, (M, K), dtype=np.int8)
    g = G.gpu_quant_weight(synth.weights(N, K, 0, "single"), 4, 128)
    q = oracle.unpack_int4(g["canon"])
    _, total, part = oracle.igemm_grouped(xq, q, g["scales"], 128, want_partials=True)
    acc, gpart = G.gpu_acc(xq, g, want_partials=True)
    assert (acc == total).all()
    assert (gpart == part).all()


# ------------------------------------------------------------------ fp16 layer
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,K,N,bias", [(64, 512, 512, False), (100, 256, 200, True), (300, 1024, 520, True),
                                        (1, 4096, 512, False), (8, 1536, 200, True), (32, 11008, 64, True),
                                        (17, 512, 33, False)])
def test_linear_fp16_within_tolerance(G, bits, M, K, N, bias):
    x = synth.activations(M, K, 0, "single")
    w = synth.weights(N, K, 0, "single")
    b = synth.bias(N, 0, "single") if bias else None
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    if bits == 8:
        ref = oracle.linear_w8a8(x, g["canon"], g["scales"], b)
    else:
        ref = oracle.linear_w4a8(x, g["canon"], g["scales"], 128, b)
    y = G.gpu_linear(x, g, b)
    assert np.isfinite(y).all()
    assert G.norm_err(y, ref["y64"]) <= TOL
    # headroom: against the un-rounded reference the error is about half an fp16 ulp of the largest value
    assert G.norm_err(y, ref["y64"]) <= 6e-4


def test_w8a8_fp16_output_has_the_same_bits_in_every_kernel(G):
    """The int32 sums are exact and every epilogue takes the same steps in the same order (one fp32 rounding per
    operation, the sum rounded to fp32 and then to fp16), so the fp16 output does not depend on the tile shape, the
    matrix instruction, split-K or the kernel family: bit-identical across all of them, and equal to those steps redone
    here in fp32 from the oracle's exact sums."""
    import torch
    M, K, N = 300, 1024, 520
    x, w, b = synth.activations(M, K, 0, "single"), synth.weights(N, K, 0, "single"), synth.bias(N, 0, "single")
    g = G.gpu_quant_weight(w, 8, 0)
    ref = oracle.linear_w8a8(x, g["canon"], g["scales"], b)
    f32 = np.float32
    t = (ref["acc"].astype(f32) * ref["sx"].astype(f32)[:, None]).astype(f32)
    # fma(t, sw, bias): one rounding of the exact t*sw + bias -- exact in the 64-bit significand of x86 long double
    # (24 x 24 bits of product plus an fp16 value a few binades below it)
    ld = np.longdouble
    assert np.finfo(ld).nmant >= 63
    want = (t.astype(ld) * g["scales"].astype(ld)[None, :] + b.astype(ld)[None, :]).astype(f32).astype(np.float16)
    outs = {}
    try:
        for variant in PREFILL_VARIANTS + [100, 104, 122, 203, 302]:
            ql.ql_set_kernel_variant(variant)
            outs[variant] = G.gpu_linear(x, g, b, extra_ws=64 << 20)
    finally:
        ql.ql_set_kernel_variant(0)
    for variant, y in outs.items():
        assert (y.view(np.uint16) == want.view(np.uint16)).all(), f"kernel variant {variant}"


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,K,N,ldx", [(1, 4096, 520, None), (2, 4096, 200, 4104), (1, 11008, 72, None), (2, 512, 33, None),
                                       (1, 128, 16, 136), (2, 8192, 48, None),
                                       (3, 4096, 200, None), (5, 4096, 520, 4104), (8, 4096, 10240, None),
                                       (8, 4096, 4608, None), (6, 4096, 72, None), (16, 1536, 4608, None),
                                       (12, 2048, 136, 2056), (7, 512, 33, None), (4, 8192, 264, None),
                                       (9, 4096, 200, None), (3, 11008, 72, None), (16, 2560, 48, None)])
def test_decode_linear_with_fused_quantization_matches_two_kernel_path(G, bits, M, K, N, ldx):
    """Few tokens (up to 16 when they fit the kernel's registers and LDS): the decode GEMM quantizes the fp16
    tokens in its prologue.  Same codes, same integer sums, same epilogue arithmetic as quantization kernel +
    GEMM, so the fp16 outputs must agree bit for bit (variant 130 forces the two-kernel path; shapes beyond the
    limits take it anyway), and both must be within tolerance of the oracle."""
    x = synth.activations(M, K, 0, "single")
    if M >= 2:
        x[1] = 0          # an all-zero token: scale 1, codes 0
    w = synth.weights(N, K, 0, "single")
    b = synth.bias(N, 0, "single")
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    y_fused = G.gpu_linear(x, g, b, ldx=ldx)
    ql.ql_set_kernel_variant(130)
    y_two = G.gpu_linear(x, g, b, ldx=ldx)
    assert (y_fused.view(np.uint16) == y_two.view(np.uint16)).all()
    ref = (oracle.linear_w8a8(x, g["canon"], g["scales"], b) if bits == 8
           else oracle.linear_w4a8(x, g["canon"], g["scales"], 128, b))
    assert G.norm_err(y_fused, ref["y64"]) <= TOL


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        bits = int(rng.choice([8, 4]))
        M = int(rng.choice([rng.integers(1, 33), rng.integers(33, 200), rng.integers(200, 700)]))
        N = int(rng.integers(1, 900))
        K = int(rng.integers(1, 33)) * 128 if bits == 4 else int(rng.integers(1, 65)) * 64   # the interface's K granularity
        out.append((bits, M, K, N, bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("bits,M,K,N,bias", _random_shapes(48, 20251223))
def test_random_shapes_with_the_automatic_kernel_choice(G, bits, M, K, N, bias):
    """Seeded random shapes (ragged in every dimension) through whatever the library picks by itself -- decode
    kernels, every prefill tile configuration, 64x64 tiles, split-K with the workspace's scratch: integer sums
    bit-exact, fp16 output within tolerance."""
    x = synth.activations(M, K, 0, "single")
    w = synth.weights(N, K, 0, "single")
    b = synth.bias(N, 0, "single") if bias else None
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    xq, _ = oracle.quant_act_per_token(x)
    acc, _ = G.gpu_acc(xq, g)
    if bits == 8:
        ref = oracle.linear_w8a8(x, g["canon"], g["scales"], b)
    else:
        ref = oracle.linear_w4a8(x, g["canon"], g["scales"], 128, b)
    assert (acc == ref["acc"]).all()
    y = G.gpu_linear(x, g, b)
    assert G.norm_err(y, ref["y64"]) <= TOL


def test_config0_end_to_end(G):
    sh = synth.workload(0)[0]
    x, w, _ = synth.tensors(sh)
    wq_o, sw_o = oracle.quant_weight_int8(w)
    ref = oracle.linear_w8a8(x, wq_o, sw_o)
    g = G.gpu_quant_weight(w, 8, 0)
    assert (g["canon"] == wq_o).all() and (g["scales"] == sw_o).all()
    y = G.gpu_linear(x, g)
    assert G.norm_err(y, ref["y64"]) <= TOL
    for v in PREFILL_VARIANTS:
        ql.ql_set_kernel_variant(v)
        assert G.norm_err(G.gpu_linear(x, g), ref["y64"]) <= TOL


def test_padded_output_is_untouched_and_runs_are_deterministic(G):
    x = synth.activations(70, 256, 0, "single")
    g = G.gpu_quant_weight(synth.weights(100, 256, 0, "single"), 8, 0)
    y1 = G.gpu_linear(x, g, ldy=112)
    y2 = G.gpu_linear(x, g, ldy=112)
    assert (y1.view(np.uint16) == y2.view(np.uint16)).all()


def test_m_zero_is_a_noop(G):
    import torch
    g = G.gpu_quant_weight(synth.weights(64, 128, 0, "single"), 8, 0)
    x = torch.empty((0, 128), dtype=torch.float16, device="cuda:0")
    y = torch.empty((0, 64), dtype=torch.float16, device="cuda:0")
    ql.ql_w8a8_linear(x, g["kernel"], g["scales_dev"].view(torch.float32), None, 64, y, None)


def test_errors_are_reported_not_launched(G):
    import torch
    g = G.gpu_quant_weight(synth.weights(64, 128, 0, "single"), 8, 0)
    x = G.dev(synth.activations(4, 128, 0, "single"))
    y = torch.empty((4, 64), dtype=torch.float16, device="cuda:0")
    with pytest.raises(ql.QlError) as e:
        ql.ql_w8a8_linear(x, g["kernel"], g["scales_dev"].view(torch.float32), None, 64, y, G.empty_bytes(16))
    assert e.value.status == 5
    with pytest.raises(ql.QlError) as e:
        ql.ql_w8a8_linear(x[:, :100], g["kernel"], g["scales_dev"].view(torch.float32), None, 64, y, G.empty_bytes(4096))
    assert e.value.status == 2


def test_kernel_variant_is_a_setting_of_the_calling_thread(G):
    """A worker thread selects split-K (which needs scratch the call does not get, so its GEMM is refused) and leaves
    that setting behind; the main thread's setting is untouched: its GEMM of the same shape runs with the automatic
    choice and matches the oracle.  Two threads with different tile variants give the same exact sums."""
    import threading
    M, K, N = 100, 1536, 264
    rng = np.random.default_rng(77)
    xq = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    g = G.gpu_quant_weight(synth.weights(N, K, 0, "single"), 8, 0)
    ref = oracle.igemm(xq, g["canon"])
    seen = {}

    def worker(name, variant):
        try:
            ql.ql_set_kernel_variant(variant)
            seen[name] = G.gpu_acc(xq, g)[0]
        except ql.QlError as e:
            seen[name] = e.status

    for name, variant in (("split", 208), ("tile13", 13), ("tile26", 26)):
        t = threading.Thread(target=worker, args=(name, variant))
        t.start()
        t.join()
    assert seen["split"] == 5                                   # QL_ERR_WORKSPACE, reported in that thread only
    assert (seen["tile13"] == ref).all() and (seen["tile26"] == ref).all()
    acc, _ = G.gpu_acc(xq, g)                                   # this thread never changed its setting
    assert (acc == ref).all()
