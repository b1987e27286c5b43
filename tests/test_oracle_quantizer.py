"""Pins for the oracle's number formats and quantizer (CPU only).

Nothing here re-types the oracle's own formula: the checks are float64 invariants that the
definition of affine min-max quantization fixes (half-step error, nearest level, end points,
constant groups, offset invariance = the asymmetric property the paper stresses in
section 7.3), exhaustive sweeps on tiny groups, and numpy / torch conversions as independent
library routines for the 16-bit formats.
"""
import numpy as np
import pytest
import torch

from util import bf16_bits_to_f64, bits_to_f64, f16_bits_to_f64, unpack_np

BITS = [2, 3, 4, 8]


# ---- number formats ------------------------------------------------------------------------

def test_f16_to_f32_all_patterns(ref):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([ref.f16_to_f32(int(b)) for b in bits], dtype=np.float32)
    fin = np.isfinite(want)
    assert np.array_equal(got[fin].view(np.uint32), want[fin].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))


def test_f32_to_f16_against_numpy(ref):
    rng = np.random.default_rng(1)
    cases = [rng.standard_normal(20000).astype(np.float32) * s for s in (1e-7, 1e-5, 1e-3, 1.0, 300.0, 7e4)]
    # every fp16 value, every midpoint between neighbours, and one float32 step either side
    h = np.arange(0x7c00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = ((h[:-1] + h[1:]) / 2).astype(np.float32)
    cases += [h.astype(np.float32), mid, np.nextafter(mid, np.float32(np.inf)),
              np.nextafter(mid, np.float32(-np.inf)), -mid,
              np.array([65504.0, 65519.99, 65520.0, 65536.0, 1e9, 0.0, -0.0, 2.0 ** -25,
                        np.nextafter(np.float32(2.0 ** -25), np.float32(1))], dtype=np.float32)]
    for x in cases:
        with np.errstate(over="ignore"):
            want = x.astype(np.float16).view(np.uint16)
        got = np.array([ref.f32_to_f16(v) for v in x], dtype=np.uint16)
        assert np.array_equal(got, want)


def test_bf16_against_torch(ref):
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0,
                        np.array([1.00390625, 1.01171875, 1.0078125, 3.3895314e38, 3.4e38, 1e-40,
                                  -0.0], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([ref.f32_to_bf16(v) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
    back = np.array([ref.bf16_to_f32(int(b)) for b in want], dtype=np.float32)
    assert np.array_equal(back.view(np.uint32), want.astype(np.uint32) << 16)


# ---- group-level invariants ----------------------------------------------------------------

def quantize_groups(ref, x_bits, dtype, bits, axis_k):
    """Run the oracle on G groups of n elements through its per-head entry point.
    x_bits: uint16 [G, n].  axis_k: groups along tokens (K) or along channels (V)."""
    G, n = x_bits.shape
    if axis_k:
        # K: tokens = n (one token block), channels = G  -> tensor [t][d] = x[d][t]
        cfg = ref.config(dtype=dtype, head_dim=G, bits_k=bits, group_k=n)
        src = np.ascontiguousarray(x_bits.T)
        lay = ref.contiguous_layout(1, n, G)
        codes, meta = ref.compress_head(cfg, 0, src, lay, n, 0, 0)
        q = unpack_np(codes, bits).reshape(n, G).T
    else:
        cfg = ref.config(dtype=dtype, head_dim=n, bits_v=bits, group_v=n)
        src = np.ascontiguousarray(x_bits)
        lay = ref.contiguous_layout(1, G, n)
        codes, meta = ref.compress_head(cfg, 1, src, lay, G, 0, 0)
        q = unpack_np(codes, bits).reshape(G, n)
    return q, meta[0::2].copy(), meta[1::2].copy()


def check_invariants(x, q, s_bits, z_bits, bits, all_levels=False):
    """x float64 [G, n]; the float64 facts every affine min-max quantizer must satisfy."""
    qmax = (1 << bits) - 1
    s = f16_bits_to_f64(s_bits)[:, None]
    z = f16_bits_to_f64(z_bits)[:, None]
    mn = x.min(axis=1, keepdims=True)
    mx = x.max(axis=1, keepdims=True)
    assert np.all(np.isfinite(s)) and np.all(s >= 0)
    assert q.max() <= qmax
    # stored metadata is the fp16 rounding of min and of range / (2^b - 1)
    s_true = (mx - mn) / qmax
    assert np.all(np.abs(s - s_true) <= np.maximum(s_true * 2.0 ** -11, 2.0 ** -25) * (1 + 1e-3))
    assert np.all(np.abs(z - mn) <= np.maximum(np.abs(mn) * 2.0 ** -11, 2.0 ** -25))
    recon = q * s + z
    err = np.abs(x - recon)
    # half a step, plus what rounding the scale can cost at the clamped top level, plus the
    # two fp32 roundings inside the quantizer
    t = np.where(s > 0, (x - z) / np.where(s > 0, s, 1), 0)
    slack = 2.0 ** -21 * (np.abs(t) + 1) * s
    bound = s / 2 + qmax * np.abs(s_true - s) + np.abs(z - mn) + slack
    assert np.all(err <= bound), float((err - bound).max())
    # nearest level: no other code is strictly closer (ties accepted)
    alts = range(qmax + 1) if all_levels else (-1, 1)
    for a in alts:
        qa = np.full_like(q, a) if all_levels else np.clip(q.astype(np.int64) + a, 0, qmax)
        assert np.all(np.abs(x - (qa * s + z)) >= err - slack)
    return recon


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("axis_k", [True, False])
def test_halfstep_and_nearest_gaussian_fp16(ref, bits, axis_k):
    rng = np.random.default_rng(10 + bits)
    x = (rng.standard_normal((4096, 32)) * rng.lognormal(size=(4096, 1))).astype(np.float16)
    q, s, z = quantize_groups(ref, x.view(np.uint16), 1, bits, axis_k)
    check_invariants(x.astype(np.float64), q, s, z, bits, all_levels=(bits <= 4))
    xs = f16_bits_to_f64(s)
    # end points: the minimum takes code 0 and reconstructs to the stored zero exactly; the
    # maximum takes the top code (scale in the normal fp16 range)
    i_mn = x.argmin(axis=1)
    i_mx = x.argmax(axis=1)
    rows = np.arange(x.shape[0])
    assert np.all(q[rows, i_mn] == 0)
    assert np.array_equal(z, x[rows, i_mn].view(np.uint16) & np.where(x[rows, i_mn] == 0, 0x7fff, 0xffff))
    ok = xs > 2.0 ** -14
    assert np.all(q[rows, i_mx][ok] == (1 << bits) - 1)


@pytest.mark.parametrize("bits", [2, 4])
def test_halfstep_bf16_input(ref, bits):
    rng = np.random.default_rng(20 + bits)
    x32 = (rng.standard_normal((2048, 64)) * 3 + 1.5).astype(np.float32)
    xb = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    q, s, z = quantize_groups(ref, xb, 2, bits, True)
    check_invariants(bf16_bits_to_f64(xb), q, s, z, bits, all_levels=True)


@pytest.mark.parametrize("bits", BITS)
def test_constant_group_is_exact(ref, bits):
    vals = np.array([0.0, -0.0, 1.0, -3.25, 65504.0, 6e-8, -1e-3], dtype=np.float16)
    x = np.repeat(vals[:, None], 32, axis=1)
    q, s, z = quantize_groups(ref, x.view(np.uint16), 1, bits, False)
    assert np.all(q == 0) and np.all(s == 0)
    assert np.array_equal(f16_bits_to_f64(z), vals.astype(np.float64))
    assert z[1] == 0                      # a zero of either sign is stored as +0
    for k in range(len(vals)):
        assert f16_bits_to_f64(ref.dequantize(0, s[k], z[k], 1)) == float(vals[k])


@pytest.mark.parametrize("bits", BITS)
def test_offset_invariance_asymmetric(ref, bits):
    """Section 7.3 blames uniform (symmetric) quantization for failing on non-zero-centred K/V.
    With an asymmetric quantizer a per-group offset must move only the zero point.  Small
    integers keep every sum exact in fp16, so the statement is exact, not approximate."""
    rng = np.random.default_rng(30 + bits)
    base = rng.integers(-8, 9, size=(512, 32)).astype(np.float64)
    base[:, 0] = -8
    base[:, 1] = 8
    off = rng.integers(-900, 901, size=(512, 1)).astype(np.float64)
    qa, sa, za = quantize_groups(ref, base.astype(np.float16).view(np.uint16), 1, bits, True)
    qb, sb, zb = quantize_groups(ref, (base + off).astype(np.float16).view(np.uint16), 1, bits, True)
    assert np.array_equal(qa, qb)
    assert np.array_equal(sa, sb)
    assert np.array_equal(f16_bits_to_f64(zb) - f16_bits_to_f64(za), off[:, 0])


@pytest.mark.parametrize("bits", BITS)
def test_exhaustive_pairs_lattice(ref, bits):
    """Every ordered pair from a 1024-value lattice of finite fp16 numbers as a 2-element group."""
    lat = np.arange(0, 0x7c00, 31, dtype=np.uint16)[:512]
    lat = np.concatenate([lat, lat | 0x8000])                # 1024 values, both signs
    a, b = np.meshgrid(lat, lat, indexing="ij")
    xb = np.stack([a.ravel(), b.ravel()], axis=1)            # [2^20, 2]
    q, s, z = quantize_groups(ref, xb, 1, bits, True)
    x = f16_bits_to_f64(xb)
    keep = np.isfinite(x).all(axis=1) & (np.abs(x[:, 0] - x[:, 1]) / ((1 << bits) - 1) < 65504)
    check_invariants(x[keep], q[keep], s[keep], z[keep], bits)


@pytest.mark.parametrize("bits", BITS)
def test_exhaustive_single_varying_element(ref, bits):
    """All 2^16 fp16 patterns as the one varying element of an otherwise fixed group of 8."""
    fixed = np.array([-1.5, 0.25, 3.0, 0.0, -0.125, 2.5, 1.0], dtype=np.float16).view(np.uint16)
    xb = np.empty((65536, 8), dtype=np.uint16)
    xb[:, :7] = fixed
    xb[:, 7] = np.arange(65536, dtype=np.uint16)
    x = f16_bits_to_f64(xb)
    keep = np.isfinite(x).all(axis=1)
    q, s, z = quantize_groups(ref, xb[keep], 1, bits, False)
    check_invariants(x[keep], q, s, z, bits)


def test_subnormal_and_tiny_ranges(ref):
    """Ranges so small that the fp16 scale is subnormal or rounds to zero: the general bound
    (half a step plus the scale's own rounding error at the top level) still holds."""
    rng = np.random.default_rng(5)
    base = rng.standard_normal((2000, 1)).astype(np.float16).astype(np.float64)
    steps = rng.integers(0, 4, size=(2000, 32))
    ulp = np.maximum(np.abs(base), 2.0 ** -14) * 2.0 ** -10
    x16 = (base + steps * ulp).astype(np.float16)
    for bits in BITS:
        q, s, z = quantize_groups(ref, x16.view(np.uint16), 1, bits, False)
        check_invariants(x16.astype(np.float64), q, s, z, bits)
    tiny = (rng.integers(-3, 4, size=(500, 32)) * 2.0 ** -24).astype(np.float16)
    for bits in BITS:
        q, s, z = quantize_groups(ref, tiny.view(np.uint16), 1, bits, True)
        check_invariants(tiny.astype(np.float64), q, s, z, bits)


def test_k_and_v_axes_are_transposes(ref):
    """K per-channel on X gives the same scales, zeros and codes as V per-token on X^T."""
    rng = np.random.default_rng(6)
    x = rng.standard_normal((64, 32)).astype(np.float16).view(np.uint16)   # 64 groups of 32
    for bits in BITS:
        qk, sk, zk = quantize_groups(ref, x, 1, bits, True)
        qv, sv, zv = quantize_groups(ref, x, 1, bits, False)
        assert np.array_equal(qk, qv) and np.array_equal(sk, sv) and np.array_equal(zk, zv)


@pytest.mark.parametrize("dtype", [1, 2])
def test_dequantize_is_rounded_affine(ref, dtype):
    """x^ = q*scale + zero rounded once to the output type: compare against exact float64
    arithmetic rounded by numpy / torch (the product and sum are exact in float64)."""
    rng = np.random.default_rng(7)
    s = rng.uniform(0, 2, 4000).astype(np.float16)
    z = (rng.standard_normal(4000) * 4).astype(np.float16)
    q = rng.integers(0, 256, 4000)
    exact = q * s.astype(np.float64) + z.astype(np.float64)
    got = np.array([ref.dequantize(int(q[i]), int(s.view(np.uint16)[i]), int(z.view(np.uint16)[i]), dtype)
                    for i in range(4000)], dtype=np.uint16)
    got64 = bits_to_f64(got, dtype)
    # nearest representable: error is at most half the gap to either neighbour
    if dtype == 1:
        want = exact.astype(np.float32).astype(np.float16)  # float32 holds q*s+z of this size exactly? no:
        # q*s+z can need more than 24 bits, so accept either float64->fp16 or the fp32-fused path
        want_direct = exact.astype(np.float16)
        ok = (got == want.view(np.uint16)) | (got == want_direct.view(np.uint16))
        assert ok.mean() > 0.999
        gap = np.abs(np.spacing(want_direct.astype(np.float16))).astype(np.float64)
        assert np.all(np.abs(got64 - exact) <= 0.5 * gap * (1 + 2.0 ** -10))
    else:
        gap = np.abs(exact) * 2.0 ** -7
        assert np.all(np.abs(got64 - exact) <= 0.5 * gap + 1e-30)
    # saturation instead of infinity at the top of the fp16 range
    top = ref.dequantize(15, 0x7044, 0xfbff, 1)            # 15 * 8736 - 65504 = 65536
    assert top == 0x7bff
