"""Pins for the oracle's delta transform (difference from an anchor token, CPU only).

Nothing here re-runs the oracle's subtraction: differences and sums are taken by numpy in float64,
where they are exact for 16-bit inputs, and rounded once by numpy's (float16) or torch's (bfloat16)
own conversions; the payload-level checks compare with payloads of the transform-free
configuration on tensors that were differenced beforehand, with closed forms for constant and
ramp inputs, and with the byte positions the anchor rows must occupy.
"""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvgen
from util import bits_to_f64, f16_bits_to_f64, unpack_np

D = 128


def to_bits(x, dtype):
    t = torch.tensor(np.asarray(x, dtype=np.float64), dtype=torch.float64)
    t = t.to(torch.float16 if dtype == 1 else torch.bfloat16)
    return kvgen.as_u16(t)


def f64_to_bits_saturating(y, dtype):
    top = 65504.0 if dtype == 1 else 3.3895313892515355e38
    y = np.clip(y, -top, top)
    if dtype == 1:
        return y.astype(np.float16).view(np.uint16)        # float64 -> float16, one rounding
    return kvgen.as_u16(torch.tensor(y, dtype=torch.float64).to(torch.bfloat16))


# ---- the row operation --------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [1, 2])
@pytest.mark.parametrize("inverse", [False, True])
def test_row_difference_is_the_exact_value_rounded_once(ref, dtype, inverse):
    rng = np.random.default_rng(20 + dtype)
    for scale in (1e-3, 1.0, 300.0):
        # a span of exponents for which the float64 sum is exact (well inside its 53 bits)
        x = to_bits(rng.standard_normal(D) * scale, dtype)
        a = to_bits(rng.standard_normal(D) * scale * rng.choice([1.0, 1 / 64.0, 64.0], D), dtype)
        xf, af = bits_to_f64(x, dtype), bits_to_f64(a, dtype)
        want = f64_to_bits_saturating(xf + af if inverse else xf - af, dtype)
        got = ref.delta_row(x, a, dtype, inverse=inverse)
        # +0 and -0: a difference of equal values is +0 in both
        assert np.array_equal(got, want), (scale, np.nonzero(got != want)[0][:5])


def test_every_pair_of_a_float16_sample_is_rounded_correctly(ref):
    """Sums whose exact value lies close to the middle between two float16 neighbours are where a
    double rounding would show: all pairs of 128 values around such cases."""
    vals = np.array([1.0, 1.0 + 2.0 ** -10, 2.0 ** -11, 3 * 2.0 ** -12, 2.0 ** -12, 2.0 ** -24, 2048.0, 2049.0 - 1.0,
                     0.5 + 2.0 ** -11, 65504.0, 33000.0, 6.1e-5, 5.96e-8, 1023.5, 0.333251953125, 4097.0])
    vals = np.concatenate([vals, -vals])
    x = np.repeat(vals, vals.size)
    a = np.tile(vals, vals.size)
    xb, ab = to_bits(x, 1), to_bits(a, 1)
    xf, af = f16_bits_to_f64(xb), f16_bits_to_f64(ab)
    for inverse in (False, True):
        want = f64_to_bits_saturating(xf + af if inverse else xf - af, 1)
        got = ref.delta_row(xb, ab, 1, inverse=inverse)
        same = (got == want) | ((f16_bits_to_f64(got) == 0) & (f16_bits_to_f64(want) == 0))
        assert same.all(), np.nonzero(~same)[0][:5]


def test_saturation_instead_of_infinity(ref):
    x = to_bits(np.full(D, 60000.0), 1)
    a = to_bits(np.full(D, -60000.0), 1)
    assert np.all(f16_bits_to_f64(ref.delta_row(x, a, 1)) == 65504.0)
    assert np.all(f16_bits_to_f64(ref.delta_row(a, x, 1)) == -65504.0)
    assert np.all(f16_bits_to_f64(ref.delta_row(x, x, 1, inverse=True)) == 65504.0)


def test_not_commutative_and_inverse_adds(ref):
    x = to_bits(np.arange(D) * 0.25, 1)
    a = to_bits(np.full(D, 3.0), 1)
    assert np.array_equal(f16_bits_to_f64(ref.delta_row(x, a, 1)), np.arange(D) * 0.25 - 3.0)
    assert np.array_equal(f16_bits_to_f64(ref.delta_row(a, x, 1)), 3.0 - np.arange(D) * 0.25)
    assert np.array_equal(f16_bits_to_f64(ref.delta_row(x, a, 1, inverse=True)), np.arange(D) * 0.25 + 3.0)


# ---- the transform in the pipeline ----------------------------------------------------------------

def differenced(x, period):
    """float64 array [..., T, D] -> rows minus the anchor row of their run (exact in float64)."""
    T = x.shape[-2]
    anchor = (np.arange(T) // period) * period
    return x - x[..., anchor, :]


@pytest.mark.parametrize("period,tokens", [(8, 72), (32, 100), (128, 300)])
def test_quantizer_sees_the_differenced_rows(ref, period, tokens):
    """Codes and metadata with the transform equal those of the transform-free configuration on a
    tensor differenced beforehand; the anchors sit in the auxiliary section, which the other
    payload does not have."""
    rng = np.random.default_rng(period)
    x = np.round(rng.standard_normal((1, 2, 2, tokens, D)) * 16.0) / 8.0       # exact differences in fp16
    y = differenced(x, period)
    xu = to_bits(x, 1).reshape(x.shape)
    yu = to_bits(y, 1).reshape(x.shape)
    assert np.array_equal(f16_bits_to_f64(yu), y)
    lay = ref.contiguous_layout(2, tokens, D)
    a = ref.compress(ref.config(heads=2, transform=2, anchor_period=period), xu[0, 0], xu[0, 1], lay, tokens)
    b = ref.compress(ref.config(heads=2), yu[0, 0], yu[0, 1], lay, tokens)
    _, _, _, _, sa = ref.inspect(a)
    _, _, _, _, sb = ref.inspect(b)
    runs = -(-tokens // period)
    assert sb[5] == 0 and sa[5] == 2 * 2 * runs * D * 2
    assert np.array_equal(a[sa[0]:sa[0] + sa[1]], b[sb[0]:sb[0] + sb[1]])       # K metadata
    assert np.array_equal(a[sa[2]:sa[2] + sa[3]], b[sb[2]:sb[2] + sb[3]])       # V metadata
    assert np.array_equal(a[sa[6]:sa[6] + sa[7]], b[sb[6]:sb[6] + sb[7]])       # K codes
    assert np.array_equal(a[sa[8]:sa[8] + sa[9]], b[sb[8]:sb[8] + sb[9]])       # V codes
    # anchors: K then V, [head][run][channel], the untouched input rows
    anchors = a[sa[4]:sa[4] + sa[5]].view(np.uint16).reshape(2, 2, runs, D)
    for kv in range(2):
        for h in range(2):
            assert np.array_equal(anchors[kv, h], xu[0, kv, h, ::period]), (kv, h)
    assert a[26] == 2 and a[28] == period and a[29] == 0 and b[28] == 0


def test_payload_size_closed_form(ref):
    for tokens, period, bits, codec in [(100, 32, 4, 0), (1, 8, 2, 0), (0, 64, 4, 0), (129, 128, 8, 1)]:
        L, H = 2, 3
        with_t = ref.config(layers=L, heads=H, bits_k=bits, bits_v=bits, codec=codec, transform=2, anchor_period=period)
        without = ref.config(layers=L, heads=H, bits_k=bits, bits_v=bits, codec=codec)
        a, _ = ref.payload_size(with_t, tokens)
        b, _ = ref.payload_size(without, tokens)
        runs = -(-tokens // period)
        aux = 512 + 4 * (2 * L * H * -(-tokens // 128) + 1) if codec else 0
        pad = (-aux) % 16
        # the anchors follow the rest of the auxiliary section from the next 16-byte boundary
        assert a - b == 2 * L * H * runs * D * 2 + (((aux + pad + 15) // 16) * 16 - ((aux + 15) // 16) * 16)


def test_constant_runs_are_lossless(ref):
    """Every row equal to its anchor: all differences are zero, all groups constant, and the
    reconstruction is the input itself at any width."""
    rng = np.random.default_rng(31)
    tokens, period = 96, 16
    base = rng.standard_normal((1, 2, 1, tokens // period, 1, D)) * 5.0
    x = np.broadcast_to(base, (1, 2, 1, tokens // period, period, D)).reshape(1, 2, 1, tokens, D)
    xu = to_bits(x, 1).reshape(x.shape)
    lay = ref.contiguous_layout(1, tokens, D)
    cfg = ref.config(bits_k=2, bits_v=2, transform=2, anchor_period=period)
    p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, tokens)
    _, _, _, _, sec = ref.inspect(p)
    assert not p[sec[6]:sec[6] + sec[7]].any() and not p[sec[8]:sec[8] + sec[9]].any()    # all codes 0
    assert not p[sec[0]:sec[0] + sec[1]].any()                                               # scale 0, zero +0
    out = np.zeros_like(xu)
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, cfg) == 0
    assert np.array_equal(out, xu)


def test_ramp_codes_in_closed_form(ref):
    """x[t] = anchor + (t mod period) * step with period = group = 16 levels apart: the K group of
    a channel holds 0, step, ..., 15 step, so at 4 bits code = t mod 16 exactly."""
    tokens, period = 64, 16
    rng = np.random.default_rng(32)
    anchor = np.round(rng.standard_normal((tokens // period, 1, D)) * 64.0)
    step = 0.5
    x = (anchor + np.arange(period).reshape(1, period, 1) * step).reshape(tokens, D)
    full = np.stack([x, x]).reshape(1, 2, 1, tokens, D)
    xu = to_bits(full, 1).reshape(full.shape)
    assert np.array_equal(f16_bits_to_f64(xu), full)
    lay = ref.contiguous_layout(1, tokens, D)
    cfg = ref.config(bits_k=4, bits_v=4, group_k=32, group_v=32, transform=2, anchor_period=period)
    p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, tokens)
    _, _, _, _, sec = ref.inspect(p)
    codes_k = unpack_np(p[sec[6]:sec[6] + sec[7]], 4).reshape(tokens, D)
    assert np.array_equal(codes_k, np.broadcast_to((np.arange(tokens) % period).reshape(-1, 1), (tokens, D)))
    # V groups lie along the channels of one token: the whole row is (t mod period) * step -> constant group
    codes_v = unpack_np(p[sec[8]:sec[8] + sec[9]], 4)
    assert not codes_v.any()
    out = np.zeros_like(xu)
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, cfg) == 0
    assert np.array_equal(out, xu)                                                           # both exact here


@pytest.mark.parametrize("dtype", [1, 2])
@pytest.mark.parametrize("codec", [0, 1])
def test_round_trip_error_bound_and_exact_anchors(ref, dtype, codec):
    """|x^ - x| <= scale/2 of the row's group in the differenced domain, plus the roundings to the
    16-bit type; anchor rows come back bit for bit."""
    tokens, period, bits = 200, 32, 4
    x = kvgen.make_kv(33, 1, 2, D, tokens, torch.float16 if dtype == 1 else torch.bfloat16)
    xu = kvgen.as_u16(x)
    lay = ref.contiguous_layout(2, tokens, D)
    cfg = ref.config(dtype=dtype, heads=2, bits_k=bits, bits_v=bits, codec=codec, transform=2, anchor_period=period)
    p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, tokens)
    out = np.zeros_like(xu)
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, cfg) == 0
    assert np.array_equal(out[:, :, :, ::period], xu[:, :, :, ::period])
    xf, of = bits_to_f64(xu, dtype), bits_to_f64(out, dtype)
    y = differenced(xf, period)
    eps = 2.0 ** -11 if dtype == 1 else 2.0 ** -8
    # K: groups of 32 tokens per channel; V: groups of 32 channels per token; range from the exact differences
    yk = y[0, 0]
    pad = (-tokens) % 32
    ykp = np.concatenate([yk, np.repeat(yk[:, -1:], pad, axis=1)], axis=1).reshape(2, -1, 32, D)
    rng_k = np.repeat(ykp.max(axis=2) - ykp.min(axis=2), 32, axis=1)[:, :tokens]
    yv = y[0, 1].reshape(2, tokens, D // 32, 32)
    rng_v = np.repeat(yv.max(axis=3) - yv.min(axis=3), 32, axis=2)
    for kv, rng_ in ((0, rng_k), (1, rng_v)):
        err = np.abs(of[0, kv] - xf[0, kv])
        scale = rng_ / (2 ** bits - 1)
        mag = np.abs(xf[0, kv]) + np.abs(y[0, kv]) + rng_
        bound = scale * (0.5 + 2.0 ** -9) + 4 * eps * mag + 1e-7
        assert np.all(err <= bound), (kv, float((err - bound).max()))


def test_differences_of_correlated_tokens_quantize_better(ref):
    """What the stage is for: when neighbouring tokens are close to each other, the per-token V
    groups of the differences span far less than those of the values."""
    rng = np.random.default_rng(34)
    tokens, period = 256, 16
    base = np.repeat(rng.standard_normal((tokens // period, 1, D)) * 4.0, period, axis=1).reshape(tokens, D)
    x = base + 0.1 * rng.standard_normal((tokens, D))
    full = np.stack([x, x]).reshape(1, 2, 1, tokens, D)
    xu = to_bits(full, 1).reshape(full.shape)
    lay = ref.contiguous_layout(1, tokens, D)
    err = {}
    for tr in (0, 2):
        cfg = ref.config(bits_k=4, bits_v=4, transform=tr, anchor_period=period if tr else 0)
        p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, tokens)
        out = np.zeros_like(xu)
        assert ref.decompress(p, out[0, 0], out[0, 1], lay, cfg) == 0
        d = f16_bits_to_f64(out[0, 1]) - f16_bits_to_f64(xu[0, 1])
        err[tr] = np.sqrt((d * d).mean())
    assert err[2] < 0.2 * err[0], err


def test_paged_equals_contiguous(ref):
    tokens, period, bt, heads = 150, 32, 16, 2
    x = kvgen.make_kv(35, 1, heads, D, tokens, torch.float16)
    xu = kvgen.as_u16(x)
    lay = ref.contiguous_layout(heads, tokens, D)
    cfg = ref.config(heads=heads, transform=2, anchor_period=period)
    want = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, tokens)
    nblk = -(-tokens // bt)
    phys = nblk + 3
    table = np.random.default_rng(1).permutation(phys)[:nblk].astype(np.int32)
    pool = np.zeros((1, 2, phys, bt, heads, D), dtype=np.uint16)
    for t in range(tokens):
        pool[0, :, table[t // bt], t % bt] = xu[0, :, :, t]
    play = ref.paged_layout(heads, D, bt, phys, table)
    got = ref.compress(cfg, pool[0, 0], pool[0, 1], play, tokens)
    assert np.array_equal(got, want)
    out = np.zeros_like(pool)
    assert ref.decompress(got, out[0, 0], out[0, 1], play, cfg) == 0
    ref_out = np.zeros_like(xu)
    assert ref.decompress(want, ref_out[0, 0], ref_out[0, 1], lay, cfg) == 0
    for t in range(tokens):
        assert np.array_equal(out[0, :, table[t // bt], t % bt], ref_out[0, :, :, t])


def test_16_bit_tensor_is_left_alone_and_carries_no_anchors(ref):
    tokens, period = 70, 8
    x = kvgen.make_kv(36, 1, 1, D, tokens, torch.float16)
    xu = kvgen.as_u16(x)
    lay = ref.contiguous_layout(1, tokens, D)
    cfg = ref.config(bits_k=16, bits_v=4, transform=2, anchor_period=period)
    p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, tokens)
    _, _, _, _, sec = ref.inspect(p)
    assert sec[5] == -(-tokens // period) * D * 2                       # V anchors only
    out = np.zeros_like(xu)
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, cfg) == 0
    assert np.array_equal(out[0, 0], xu[0, 0])


def test_config_errors(ref):
    for period in (0, 4, 12, 256):
        with pytest.raises(ValueError):
            ref.payload_size(ref.config(transform=2, anchor_period=period), 10)
    with pytest.raises(ValueError):
        ref.payload_size(ref.config(transform=0, anchor_period=32), 10)
    with pytest.raises(ValueError):
        ref.payload_size(ref.config(transform=3), 10)


def test_decompress_rejects_a_changed_period(ref):
    tokens = 64
    x = kvgen.make_kv(37, 1, 1, D, tokens, torch.float16)
    xu = kvgen.as_u16(x)
    lay = ref.contiguous_layout(1, tokens, D)
    cfg = ref.config(transform=2, anchor_period=32)
    p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, tokens)
    out = np.zeros_like(xu)
    other = ref.config(transform=2, anchor_period=16)
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, other) == -5          # mismatch with the expectation
    bad = p.copy()
    bad[28] = 16                                                             # sizes no longer fit the header
    assert ref.decompress(bad, out[0, 0], out[0, 1], lay, None) == -4
    bad = p.copy()
    bad[30] = 1
    assert ref.decompress(bad, out[0, 0], out[0, 1], lay, None) == -4
