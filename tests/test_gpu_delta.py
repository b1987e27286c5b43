"""GPU parity for the delta transform (run with -m gpu): payload bytes, anchors included, and
reconstructions of the HIP path against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvc, kvgen
from test_gpu_parity import check_contiguous, first_diff, gpu_compress

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("bits,group,period", [(4, 32, 32), (2, 64, 64), (3, 128, 32), (8, 32, 128), (4, 128, 64),
                                               (4, 32, 8), (3, 64, 16), (2, 128, 8), (8, 32, 16)])
def test_delta_contiguous(ref, dtype, bits, group, period):
    x = kvgen.make_kv(80 + bits, 2, 2, 128, 32 * 9 + 5, dtype)
    check_contiguous(ref, x, bits, bits, group, group, transform=2, anchor_period=period)


@pytest.mark.parametrize("T", [1, 7, 8, 9, 31, 33, 129])
def test_delta_short_sequences(ref, T):
    x = kvgen.make_kv(81, 1, 2, 128, T, torch.float16)
    check_contiguous(ref, x, 4, 4, 32, 32, transform=2, anchor_period=64)
    check_contiguous(ref, x, 4, 4, 32, 32, transform=2, anchor_period=32)


@pytest.mark.parametrize("period", [8, 16, 32, 64, 128])
def test_delta_with_codec_and_ragged_tail(ref, period):
    x = kvgen.make_kv(82, 2, 4, 128, 128 * 5 + 37, torch.float16)
    check_contiguous(ref, x, 4, 4, 32, 32, codec=1, transform=2, anchor_period=period)
    check_contiguous(ref, x, 4, 2, 64, 64, codec=1, transform=2, anchor_period=period, T=128 * 3 + 1)


def test_delta_codec_bf16_8_bits(ref):
    x = kvgen.make_kv(83, 1, 3, 128, 128 * 4 + 3, torch.bfloat16)
    check_contiguous(ref, x, 8, 8, 32, 32, codec=1, transform=2, anchor_period=64)


def test_delta_mixed_with_passthrough(ref):
    """A tensor stored unchanged is not differenced and carries no anchors; the other one is."""
    x = kvgen.make_kv(84, 1, 2, 128, 100, torch.float16)
    check_contiguous(ref, x, 16, 4, 32, 32, transform=2, anchor_period=32)
    check_contiguous(ref, x, 4, 16, 32, 32, transform=2, anchor_period=32)


def test_delta_tokens_shorter_than_allocation(ref):
    x = kvgen.make_kv(85, 2, 2, 128, 300, torch.float16)
    check_contiguous(ref, x, 4, 4, 32, 32, transform=2, anchor_period=32, T=211)


def test_delta_saturates_instead_of_overflowing(ref):
    x = torch.full((1, 2, 1, 64, 128), 60000.0, dtype=torch.float16)
    x[0, :, 0, 1::2] = -60000.0
    check_contiguous(ref, x, 4, 4, 32, 32, transform=2, anchor_period=32)
    check_contiguous(ref, x, 8, 8, 32, 32, transform=2, anchor_period=128)


def test_delta_correlated_tokens(ref):
    """Token-correlated data (what the stage is for): small differences around large anchors."""
    g = torch.Generator().manual_seed(86)
    base = torch.randn(2, 2, 2, 10, 1, 128, generator=g) * 6.0
    x = (base + 0.05 * torch.randn(2, 2, 2, 10, 32, 128, generator=g)).reshape(2, 2, 2, 320, 128).to(torch.float16)
    check_contiguous(ref, x, 2, 2, 32, 32, transform=2, anchor_period=32)
    check_contiguous(ref, x, 4, 4, 32, 32, codec=1, transform=2, anchor_period=32)


def test_delta_paged(ref):
    L, H, bt, P, T = 2, 2, 16, 24, 16 * 13 + 7
    for codec in (0, 1):
        cfg = ref.config(dtype=1, layers=L, heads=H, bits_k=4, bits_v=4, group_k=32, group_v=32, codec=codec,
                         transform=2, anchor_period=32)
        plan = kvc.Plan(1, L, H, 128, 4, 4, 32, 32, codec, max_tokens=T, transform=2, anchor_period=32)
        x = kvgen.make_kv(87, L, H, 128, T, torch.float16)
        tab = kvgen.block_table(5, -(-T // bt), P)
        pool = kvgen.to_paged(x, tab, bt, P).cuda()
        tabd = tab.cuda()
        buf = gpu_compress(plan, [kvc.paged_request(pool, tabd, T)], [T])
        xu = kvgen.as_u16(x)
        lay = ref.contiguous_layout(H, T, 128)
        want = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, T)
        got = buf.payload_of(0)
        assert int(buf.status[0]) == 0
        assert np.array_equal(got, want), first_diff(got, want)
        out = torch.zeros_like(pool)
        buf.decompress([kvc.paged_request(out, tabd, T)], torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert int(buf.status[0]) == 0
        y = kvgen.from_paged(out.cpu(), tab, T)
        ru = np.zeros_like(xu)
        assert ref.decompress(want, ru[0, 0], ru[0, 1], lay, cfg) == 0
        assert np.array_equal(kvgen.as_u16(y), ru)


def test_delta_with_per_head_widths(ref):
    L, H, T = 2, 4, 200
    rng = np.random.default_rng(88)
    tk = rng.choice([2, 3, 4, 8], L * H).astype(np.uint8)
    tv = rng.choice([2, 8], L * H).astype(np.uint8)
    x = kvgen.make_kv(88, L, H, 128, T, torch.float16)
    xu = kvgen.as_u16(x)
    cfg = ref.config(dtype=1, layers=L, heads=H, group_k=32, group_v=32, transform=2, anchor_period=64,
                     head_bits_k=tk, head_bits_v=tv)
    lay = ref.contiguous_layout(H, T, 128)
    want = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, T)
    plan = kvc.Plan(1, L, H, 128, 0, 0, 32, 32, 0, max_tokens=T, transform=2, anchor_period=64,
                    head_bits_k=tk, head_bits_v=tv)
    xd = x.cuda()
    buf = gpu_compress(plan, [kvc.contiguous_request(xd, T)], [T])
    assert int(buf.status[0]) == 0
    got = buf.payload_of(0)
    assert np.array_equal(got, want), first_diff(got, want)
    y = torch.zeros_like(xd)
    buf.decompress([kvc.contiguous_request(y, T)], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert int(buf.status[0]) == 0
    ru = np.zeros_like(xu)
    assert ref.decompress(want, ru[0, 0], ru[0, 1], lay, cfg) == 0
    assert np.array_equal(kvgen.as_u16(y.cpu()), ru)


def test_delta_period_mismatch_is_reported(ref):
    T = 96
    x = kvgen.make_kv(89, 1, 2, 128, T, torch.float16).cuda()
    plan = kvc.Plan(1, 1, 2, 128, 4, 4, 32, 32, 0, max_tokens=T, transform=2, anchor_period=32)
    buf = gpu_compress(plan, [kvc.contiguous_request(x, T)], [T])
    buf.payload[28] = 64                                # the header now names another period
    y = torch.zeros_like(x)
    buf.decompress([kvc.contiguous_request(y, T)], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert int(buf.status[0]) & kvc.DEV_BAD_HEADER
    assert not y.any()                                  # nothing was written


@pytest.mark.parametrize("period", [8, 16])
def test_delta_short_runs(ref, period):
    """Runs of 8 and 16 tokens (several anchors per pass of 32 rows): ragged ends inside and between
    runs, paged pools, the lossless stage, and both types."""
    for T in (1, 7, 8, 9, 15, 16, 17, 24, 25, 33, 40, 129):
        x = kvgen.make_kv(84, 1, 2, 128, T, torch.float16)
        check_contiguous(ref, x, 4, 4, 32, 32, transform=2, anchor_period=period)
    x = kvgen.make_kv(85, 2, 2, 128, 128 * 2 + 21, torch.bfloat16)
    check_contiguous(ref, x, 4, 2, 64, 64, codec=1, transform=2, anchor_period=period)
    check_contiguous(ref, x, 8, 3, 128, 32, transform=2, anchor_period=period, T=100)


@pytest.mark.parametrize("codec", [0, 1])
def test_delta_ragged_batch(ref, codec):
    """A batch of requests of different lengths (one empty): every payload, with its own anchor
    rows, equals the one the oracle makes for that request alone."""
    L, H = 2, 4
    lens = [70, 128, 0, 201, 33]
    cfg = ref.config(dtype=2, layers=L, heads=H, bits_k=4, bits_v=2, group_k=64, group_v=64, codec=codec,
                     transform=2, anchor_period=32)
    plan = kvc.Plan(2, L, H, 128, 4, 2, 64, 64, codec, max_tokens=max(lens), max_batch=len(lens), transform=2,
                    anchor_period=32)
    xs = [kvgen.make_kv(110 + i, L, H, 128, max(T, 1), torch.bfloat16) for i, T in enumerate(lens)]
    xd = [x.cuda() for x in xs]
    buf = gpu_compress(plan, [kvc.contiguous_request(x, T) for x, T in zip(xd, lens)], lens)
    for i, T in enumerate(lens):
        xu = kvgen.as_u16(xs[i])
        want = ref.compress(cfg, xu[0, 0], xu[0, 1], ref.contiguous_layout(H, max(T, 1), 128), T)
        assert int(buf.status[i]) == 0
        got = buf.payload_of(i)
        assert np.array_equal(got, want), (i, first_diff(got, want))
    ys = [torch.zeros_like(x) for x in xd]
    buf.decompress([kvc.contiguous_request(y, T) for y, T in zip(ys, lens)], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for i, T in enumerate(lens):
        xu = kvgen.as_u16(xs[i])
        ru = np.zeros_like(xu)
        assert ref.decompress(buf.payload_of(i), ru[0, 0], ru[0, 1], ref.contiguous_layout(H, max(T, 1), 128), cfg) == 0
        assert np.array_equal(kvgen.as_u16(ys[i].cpu()), ru), i
