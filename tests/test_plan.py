"""Host logic of the automatic kernel choice, through ql_plan_gemm (no GPU call is made)."""
import ctypes
import math

import pytest

from paper_2512_23367_amd import binding as ql

SCRATCH = 64 << 20


def plan(M, N, K, bits=8, scratch=SCRATCH):
    return ql.ql_plan_gemm(M, N, K, bits, 0 if bits == 8 else 128, scratch)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M", [1, 4, 16, 17, 32])
@pytest.mark.parametrize("N,K", [(1536, 1536), (4096, 4096), (22016, 4096), (4096, 11008), (33, 128)])
def test_up_to_32_tokens_always_take_the_decode_kernels(bits, M, N, K):
    p = plan(M, N, K, bits)
    assert p.family == ql.QL_FAMILY_DECODE and p.splits == 1
    assert p.tile_tokens == (16 if M <= 16 else 32)
    assert p.tile_channels in (16, 32, 48, 64) and p.variant == 100 + p.tile_channels // 16
    # launch + the weight stream at 7.2 TB/s
    assert p.est_us == pytest.approx(3.5 + N * K * bits / 8 / 7.2e6)


def test_few_tokens_on_7b_shapes_follow_the_measured_table():
    """64 tokens: every 7B projection goes to the decode kernels; the small-N ones in blocks of 32 tokens x 32
    channels, the others in blocks of 64 with as many channel groups as fit the workgroups into one pass."""
    for N, K, block, channels in [(4096, 4096, 32, 32), (4096, 11008, 32, 32), (12288, 4096, 64, 48), (22016, 4096, 64, 96)]:
        p = plan(64, N, K)
        assert (p.family, p.tile_tokens, p.tile_channels) == (ql.QL_FAMILY_DECODE, block, channels), (N, K)
        groups = -(-N // 32) * 2
        assert -(-groups // (channels // 16)) * -(-64 // block) <= 256          # one pass over the 256 CUs
    # int4 weights have C <= 4: the widest projection needs two passes and still beats the one int4 tile shape
    p = plan(64, 22016, 4096, bits=4)
    assert p.family == ql.QL_FAMILY_DECODE and p.tile_channels <= 64


def test_config1_prefill_shapes_take_the_profiled_tile_kernels():
    for N, K, variant, tile in [(4608, 1536, 35, (256, 192)), (1536, 1536, 13, (128, 128)), (12288, 1536, 43, (256, 384)),
                                (1536, 6144, 39, (128, 128))]:
        p = plan(2048, N, K)
        assert (p.family, p.variant, (p.tile_tokens, p.tile_channels), p.splits) == (ql.QL_FAMILY_TILE, variant, tile, 1)


@pytest.mark.parametrize("bits", [8, 4])
def test_beyond_1024_tokens_only_tile_kernels(bits):
    for M in (1025, 2048, 16384):
        for N, K in [(1536, 1536), (4096, 4096), (128, 128)]:
            assert plan(M, N, K, bits).family == ql.QL_FAMILY_TILE


def test_split_k_needs_scratch_and_fits_it():
    M, N, K = 128, 4096, 11008
    with_scratch = plan(M, N, K, scratch=SCRATCH)
    assert with_scratch.family == ql.QL_FAMILY_TILE and with_scratch.splits > 1
    assert with_scratch.variant == (200 if with_scratch.tile_tokens == 128 else 300) + with_scratch.splits
    tiles = -(-M // with_scratch.tile_tokens) * -(-N // with_scratch.tile_channels)
    assert with_scratch.splits * tiles * with_scratch.tile_tokens * with_scratch.tile_channels * 4 <= SCRATCH
    without = plan(M, N, K, scratch=0)
    assert without.splits == 1
    small = plan(M, N, K, scratch=1 << 20)      # room for no split of this shape
    assert small.splits == 1
    # the int4 kernel splits too, and reports the variant that selects the same split
    p4 = plan(200, 4096, 11008, bits=4)
    if p4.family == ql.QL_FAMILY_TILE and p4.splits > 1:
        assert p4.variant == 200 + p4.splits


def test_estimates_are_finite_positive_and_grow_with_k():
    for M in (1, 64, 300, 2048):
        last = 0.0
        for K in (512, 1024, 2048, 4096, 8192, 16384):
            p = plan(M, 4096, K)
            assert math.isfinite(p.est_us) and p.est_us > 2.0
            assert p.est_us >= last * 0.999, (M, K)
            last = p.est_us


def test_the_choice_is_the_lower_estimate():
    """Between 33 and 1024 tokens the family with the lower estimate is taken: forcing more work onto one of them
    (longer K leaves the ratio alone, but more tokens favour the tiles) eventually flips the choice, once."""
    fams = [plan(M, 12288, 4096).family for M in (33, 64, 128, 256, 512, 1024)]
    assert fams[0] == ql.QL_FAMILY_DECODE and fams[-1] == ql.QL_FAMILY_TILE
    flips = sum(a != b for a, b in zip(fams, fams[1:]))
    assert flips == 1


def test_int4_with_very_long_k_cannot_stage_its_scales_and_takes_the_tiles():
    assert plan(64, 256, 131072, bits=4).family == ql.QL_FAMILY_TILE
    assert plan(8, 256, 131072, bits=4).family == ql.QL_FAMILY_DECODE     # up to 32 tokens: always


def test_argument_errors():
    lib = ql.lib()
    p = ql.QlPlan()
    assert lib.ql_plan_gemm(64, 128, 128, 8, 0, 0, None) == 1                      # QL_ERR_NULL
    assert lib.ql_plan_gemm(0, 128, 128, 8, 0, 0, ctypes.byref(p)) == 2            # QL_ERR_SHAPE
    assert lib.ql_plan_gemm(64, 128, 100, 8, 0, 0, ctypes.byref(p)) == 2           # K granularity
    assert lib.ql_plan_gemm(64, 128, 128, 8, 128, 0, ctypes.byref(p)) == 4         # unsupported (bits, group)
    assert lib.ql_plan_gemm(64, 128, 128, 8, 0, 0, ctypes.byref(p)) == 0


def test_channel_split_only_where_whole_passes_are_left_partly_filled():
    """7B gate+up at 4096 tokens: 928 tiles of 256x384 are 3.6 passes over 256 CUs; the plan runs 3 whole passes
    (18432 channels) and gives the remaining 3584 channels to 256x256 tiles (224 of them, one pass).  Shapes whose tiles
    already make whole passes, few-token shapes and int4 weights keep one launch."""
    p = plan(4096, 22016, 4096)
    assert (p.variant, p.tile_channels, p.rest_channels, p.rest_variant, p.splits) == (43, 384, 3584, 26, 1)
    assert (22016 - p.rest_channels) % 384 == 0 and (4096 // 256) * ((22016 - p.rest_channels) // 384) % 256 == 0
    for M, N, K in [(4096, 12288, 4096), (4096, 4096, 4096), (4096, 4096, 11008), (2048, 12288, 1536), (2048, 4608, 1536)]:
        assert plan(M, N, K).rest_channels == 0
    assert plan(1024, 22016, 4096).rest_channels == 0
    assert plan(4096, 22016, 4096, bits=4).rest_channels == 0
    assert plan(32, 22016, 4096).rest_channels == 0


def test_channel_split_is_taken_only_for_a_lower_estimate_and_keeps_channel_blocks_whole():
    for M, N, K in [(4096, 22016, 4096), (16384, 4096, 11008), (4096, 13824, 5120), (1100, 21767, 2048), (2048, 12289, 2048)]:
        p = plan(M, N, K)
        assert p.rest_channels > 0 and p.rest_variant > 0
        first = N - p.rest_channels
        assert first > 0 and first % p.tile_channels == 0          # whole tiles, hence whole 32-channel row-blocks
        # the estimate is the sum of the two launches' own estimates (scratch is not shared between them)
        assert p.est_us <= 1.0001 * (plan(M, first, K, scratch=0).est_us + plan(M, p.rest_channels, K, scratch=0).est_us)
