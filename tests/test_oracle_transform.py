"""Pins for the oracle's transform stage T (Walsh-Hadamard over head_dim, CPU only).

The checks do not re-run the oracle's butterfly: they compare it with the matrix definition
H[i][j] = (-1)^popcount(i & j) evaluated by numpy in integers or float64 (exact for the inputs
used), with the columns of H for unit impulses, with the identity that the forward / inverse pair
must form, with an energy identity, and with one hand-computed case in which the order of the
fp32 additions decides the result.
"""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvgen
from util import bf16_bits_to_f64, bits_to_f64, f16_bits_to_f64, ulp_distance_16

D = 128


def hadamard_matrix(n):
    i = np.arange(n)
    pop = np.array([[bin(a & b).count("1") for b in i] for a in i])
    return np.where(pop % 2 == 0, 1, -1).astype(np.int64)


H = hadamard_matrix(D)


def to_bits(x, dtype):
    t = torch.tensor(np.asarray(x, dtype=np.float64), dtype=torch.float64)
    t = t.to(torch.float16 if dtype == 1 else torch.bfloat16)
    return kvgen.as_u16(t)


@pytest.mark.parametrize("dtype", [1, 2])
def test_unit_impulses_give_the_columns_of_h(ref, dtype):
    for k in [0, 1, 2, 5, 64, 77, 127]:
        x = np.zeros(D)
        x[k] = 8.0
        y = bits_to_f64(ref.hadamard_row(to_bits(x, dtype), dtype), dtype)
        assert np.array_equal(y, H[:, k].astype(np.float64)), k            # forward scale 1/8
        z = bits_to_f64(ref.hadamard_row(to_bits(x, dtype), dtype, inverse=True), dtype)
        assert np.array_equal(z, H[:, k] * 0.5), k                          # inverse scale 1/16


@pytest.mark.parametrize("dtype,span", [(1, 8), (2, 1)])
def test_small_integers_are_transformed_exactly(ref, dtype, span):
    """Inputs that are multiples of 8: every sum is an integer far below 2^11 (2^8 for bfloat16),
    so nothing rounds and the result must equal the integer matrix product."""
    rng = np.random.default_rng(3)
    for _ in range(50):
        x = rng.integers(-span, span + 1, D) * 8
        y = bits_to_f64(ref.hadamard_row(to_bits(x, dtype), dtype), dtype)
        assert np.array_equal(y, (H @ x) / 8.0)
        back = bits_to_f64(ref.hadamard_row(to_bits(y, dtype), dtype, inverse=True), dtype)
        assert np.array_equal(back, x.astype(np.float64))                   # (H/8)(H/16) = I


@pytest.mark.parametrize("dtype", [1, 2])
def test_against_float64_definition(ref, dtype):
    rng = np.random.default_rng(4)
    eps16 = 2.0 ** -11 if dtype == 1 else 2.0 ** -8        # half an ulp, relative
    for scale in (1e-3, 1.0, 40.0):
        x = bits_to_f64(to_bits(rng.standard_normal(D) * scale, dtype), dtype)
        for inverse, s in ((False, 8.0), (True, 16.0)):
            y = bits_to_f64(ref.hadamard_row(to_bits(x, dtype), dtype, inverse=inverse), dtype)
            want = (H @ x) / s
            # one rounding to the 16-bit type plus the fp32 rounding of at most 7 additions
            bound = eps16 * np.abs(want) * 1.001 + 8 * 2.0 ** -24 * np.abs(x).sum() / s + 2.0 ** -25
            assert np.all(np.abs(y - want) <= bound), (scale, inverse)


def test_energy_identity(ref):
    rng = np.random.default_rng(5)
    x = f16_bits_to_f64(to_bits(rng.standard_normal(D), 1))
    y = f16_bits_to_f64(ref.hadamard_row(to_bits(x, 1), 1))
    assert abs((y * y).sum() / (2.0 * (x * x).sum()) - 1.0) < 2e-3            # |Hx/8|^2 = 2 |x|^2


def test_round_trip_is_close_to_identity(ref):
    rng = np.random.default_rng(6)
    for dtype, tol in ((1, 2.0 ** -9), (2, 2.0 ** -6)):
        x = bits_to_f64(to_bits(rng.standard_normal(D) * 3.0, dtype), dtype)
        y = ref.hadamard_row(to_bits(x, dtype), dtype)
        z = bits_to_f64(ref.hadamard_row(y, dtype, inverse=True), dtype)
        assert np.abs(z - x).max() <= tol * np.abs(x).max() * 4


def test_saturation_instead_of_infinity(ref):
    x = np.full(D, 65504.0)
    y = ref.hadamard_row(to_bits(x, 1), 1)
    assert y[0] == 0x7bff and not np.any(y[1:] & 0x7fff)                      # 128 * 65504 / 8 saturates
    y = ref.hadamard_row(to_bits(-x, 1), 1)
    assert y[0] == 0xfbff


def test_addition_order_is_stride_1_first(ref):
    """8192 + 2^-11 is not representable in fp32 (25 significant bits).  With the strides taken in
    the order 1, 2, 4, ... the two large entries cancel in the first stage (index 0 and 1), the two
    small ones add up exactly (index 64 and 65), and output 0 = (0 + 2 * 2^-11) / 8 = 2^-13.  Taking
    stride 64 first would add 2^-11 to +-8192, lose it, and give 0."""
    x = np.zeros(D)
    x[0], x[1], x[64], x[65] = 8192.0, -8192.0, 2.0 ** -11, 2.0 ** -11
    y = f16_bits_to_f64(ref.hadamard_row(to_bits(x, 1), 1))
    assert y[0] == 2.0 ** -13
    # output 1 = (x0 - x1 + x64 - x65) / 8 = 2048, reached without rounding
    assert y[1] == 2048.0


# ---- T in the pipeline -------------------------------------------------------------------------

def test_header_and_sizes_with_transform(ref):
    x = kvgen.make_kv(11, 1, 2, D, 96, torch.float16)
    xu = kvgen.as_u16(x)
    lay = ref.contiguous_layout(2, 96, D)
    plain = ref.compress(ref.config(layers=1, heads=2), xu[0, 0], xu[0, 1], lay, 96)
    rot = ref.compress(ref.config(layers=1, heads=2, transform=1), xu[0, 1 - 1], xu[0, 1], lay, 96)
    assert plain.size == rot.size                       # T adds no bytes
    assert plain[26] == 0 and rot[26] == 1
    rc, cfg, tokens, total, sec = ref.inspect(rot)
    assert rc == 0 and cfg.transform == 1 and tokens == 96


def test_identity_at_16_bits_survives_the_transform(ref):
    x = kvgen.make_kv(12, 1, 2, D, 40, torch.float16)
    xu = kvgen.as_u16(x)
    lay = ref.contiguous_layout(2, 40, D)
    cfg = ref.config(layers=1, heads=2, bits_k=16, bits_v=16, transform=1)
    p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, 40)
    out = np.zeros_like(xu)
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, cfg) == 0
    assert np.array_equal(out, xu)


def test_quantizer_sees_the_transformed_rows(ref):
    """Codes and metadata of a payload with T equal those of a payload without T computed on rows
    that were transformed beforehand (by the float64 definition, which is exact for these inputs)."""
    rng = np.random.default_rng(7)
    T = 64
    x = rng.integers(-3, 4, (1, 2, 1, T, D)) * 8.0
    y = np.einsum("ij,...j->...i", H.astype(np.float64), x) / 8.0
    xu = to_bits(x, 1).reshape(1, 2, 1, T, D)
    yu = to_bits(y, 1).reshape(1, 2, 1, T, D)
    lay = ref.contiguous_layout(1, T, D)
    a = ref.compress(ref.config(transform=1), xu[0, 0], xu[0, 1], lay, T)
    b = ref.compress(ref.config(transform=0), yu[0, 0], yu[0, 1], lay, T)
    assert np.array_equal(a[128:], b[128:])
    assert np.array_equal(np.nonzero(a[:128] != b[:128])[0], [26])


def test_rotation_spreads_an_outlier_channel(ref):
    """The reason the stage exists: one large channel inside a per-token group costs every other
    channel of the group its resolution; after the rotation no single coordinate dominates."""
    rng = np.random.default_rng(8)
    T = 128
    v = rng.standard_normal((T, D))
    v[:, 17] *= 30.0
    x = np.zeros((1, 2, 1, T, D))
    x[0, 0, 0] = rng.standard_normal((T, D))
    x[0, 1, 0] = v
    xu = to_bits(x, 1).reshape(1, 2, 1, T, D)
    lay = ref.contiguous_layout(1, T, D)
    err = {}
    for tr in (0, 1):
        cfg = ref.config(bits_k=4, bits_v=4, group_k=32, group_v=128, transform=tr)
        p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, T)
        out = np.zeros_like(xu)
        assert ref.decompress(p, out[0, 0], out[0, 1], lay, cfg) == 0
        d = f16_bits_to_f64(out[0, 1, 0]) - f16_bits_to_f64(xu[0, 1, 0])
        err[tr] = np.sqrt((d * d).mean())
    assert err[1] < 0.5 * err[0], err
