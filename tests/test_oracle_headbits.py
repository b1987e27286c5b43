"""Pins for per-head bit widths in the oracle (CPU only).  The mixed payload is checked against
payloads with one uniform width, which the other oracle tests pin: every head of the mixed payload
must carry exactly the metadata and codes that the uniform payload of its width carries for it, in
(layer, head) order, and must reconstruct to the same values."""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvgen

L, H, D, T = 3, 4, 128, 70
WIDTHS = [2, 3, 4, 8]


def a16(n):
    return (n + 15) // 16 * 16


@pytest.fixture(scope="module")
def data():
    x = kvgen.make_kv(21, L, H, D, T, torch.float16)
    return kvgen.as_u16(x)


def tables(seed):
    rng = np.random.default_rng(seed)
    return rng.choice(WIDTHS, L * H).astype(np.uint8), rng.choice(WIDTHS, L * H).astype(np.uint8)


@pytest.mark.parametrize("transform", [0, 1])
def test_every_head_equals_its_uniform_payload(ref, data, transform):
    tk, tv = tables(1)
    lay = ref.contiguous_layout(H, T, D)
    cfg = ref.config(layers=L, heads=H, group_k=32, group_v=64, head_bits_k=tk, head_bits_v=tv, transform=transform)
    mixed = ref.compress(cfg, data[0, 0], data[0, 1], lay, T)
    rc, _, tokens, total, sec = ref.inspect(mixed)
    assert rc == 0 and tokens == T and total == mixed.size
    out = np.zeros_like(data)
    assert ref.decompress(mixed, out[0, 0], out[0, 1], lay, cfg) == 0
    uniform = {}
    for b in WIDTHS:
        c = ref.config(layers=L, heads=H, bits_k=b, bits_v=b, group_k=32, group_v=64, transform=transform)
        p = ref.compress(c, data[0, 0], data[0, 1], lay, T)
        o = np.zeros_like(data)
        assert ref.decompress(p, o[0, 0], o[0, 1], lay, c) == 0
        uniform[b] = (p, ref.inspect(p)[4], o)
    nbk = -(-T // 32)
    meta_head = [4 * nbk * D, 4 * T * (D // 64)]
    for is_v, tab in ((0, tk), (1, tv)):
        off = 0
        for lh in range(L * H):
            b = int(tab[lh])
            p, s, o = uniform[b]
            hb = T * D * b // 8
            got = mixed[sec[6 + 2 * is_v] + off: sec[6 + 2 * is_v] + off + hb]
            want = p[s[6 + 2 * is_v] + lh * hb: s[6 + 2 * is_v] + (lh + 1) * hb]
            assert np.array_equal(got, want), (is_v, lh)
            m = meta_head[is_v]
            assert np.array_equal(mixed[sec[2 * is_v] + lh * m: sec[2 * is_v] + (lh + 1) * m],
                                  p[s[2 * is_v] + lh * m: s[2 * is_v] + (lh + 1) * m]), (is_v, lh)
            l, h = divmod(lh, H)
            assert np.array_equal(out[l, is_v, h], o[l, is_v, h]), (is_v, lh)
            off += hb
        assert off == sec[7 + 2 * is_v]


def test_size_closed_form_and_tables_in_the_payload(ref, data):
    tk, tv = tables(2)
    lay = ref.contiguous_layout(H, T, D)
    cfg = ref.config(layers=L, heads=H, group_k=32, group_v=32, head_bits_k=tk, head_bits_v=tv)
    p = ref.compress(cfg, data[0, 0], data[0, 1], lay, T)
    meta_k, meta_v = 4 * L * H * -(-T // 32) * D, 4 * L * H * T * (D // 32)
    codes_k, codes_v = int(T * D * tk.astype(int).sum() // 8), int(T * D * tv.astype(int).sum() // 8)
    assert p.size == 128 + a16(meta_k) + a16(meta_v) + a16(2 * L * H) + a16(codes_k) + a16(codes_v)
    assert ref.payload_size(cfg, T)[0] == p.size
    rc, _, _, _, sec = ref.inspect(p)
    assert sec[5] == 2 * L * H
    assert np.array_equal(p[sec[4]: sec[4] + L * H], tk) and np.array_equal(p[sec[4] + L * H: sec[4] + 2 * L * H], tv)
    assert p[20] == 0 and p[21] == 0 and p[27] == 3


def test_constant_table_is_the_uniform_case(ref, data):
    lay = ref.contiguous_layout(H, T, D)
    only_k = ref.config(layers=L, heads=H, bits_v=4, head_bits_k=np.full(L * H, 3, np.uint8))
    a = ref.compress(only_k, data[0, 0], data[0, 1], lay, T)
    b = ref.compress(ref.config(layers=L, heads=H, bits_k=3, bits_v=4), data[0, 0], data[0, 1], lay, T)
    sa, sb = ref.inspect(a)[4], ref.inspect(b)[4]
    assert a[27] == 1 and a[20] == 0 and a[21] == 4 and sa[5] == L * H and sb[5] == 0
    for i in (0, 2, 6, 8):                              # K meta, V meta, K codes, V codes
        assert np.array_equal(a[sa[i]: sa[i] + sa[i + 1]], b[sb[i]: sb[i] + sb[i + 1]])


def test_half_step_bound_per_head(ref, data):
    tk, tv = tables(3)
    lay = ref.contiguous_layout(H, T, D)
    cfg = ref.config(layers=L, heads=H, group_k=32, group_v=32, head_bits_k=tk, head_bits_v=tv)
    p = ref.compress(cfg, data[0, 0], data[0, 1], lay, T)
    out = np.zeros_like(data)
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, cfg) == 0
    sec = ref.inspect(p)[4]
    x = data.view(np.float16).astype(np.float64)
    y = out.view(np.float16).astype(np.float64)
    vmeta = p[sec[2]: sec[2] + sec[3]].view(np.float16).astype(np.float64).reshape(L, H, T, D // 32, 2)
    for l in range(L):
        for h in range(H):
            scale = np.repeat(vmeta[l, h, :, :, 0], 32, axis=1)
            assert np.all(np.abs(x[l, 1, h] - y[l, 1, h]) <= scale / 2 * 1.002 + 1e-3 * np.abs(x[l, 1, h]) + 1e-6)


def test_rejections(ref, data):
    lay = ref.contiguous_layout(H, T, D)
    tk, tv = tables(4)
    bad = tk.copy()
    bad[5] = 5
    with pytest.raises(ValueError):
        ref.compress(ref.config(layers=L, heads=H, head_bits_k=bad), data[0, 0], data[0, 1], lay, T)
    with pytest.raises(ValueError):
        ref.compress(ref.config(layers=L, heads=H, head_bits_k=tk, codec=1), data[0, 0], data[0, 1], lay, T)
    cfg = ref.config(layers=L, heads=H, head_bits_k=tk, head_bits_v=tv)
    p = ref.compress(cfg, data[0, 0], data[0, 1], lay, T)
    out = np.zeros_like(data)
    other = tk.copy()
    other[0] = 2 if tk[0] != 2 else 4
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, ref.config(layers=L, heads=H, head_bits_k=other, head_bits_v=tv)) == -5
    assert ref.decompress(p, out[0, 0], out[0, 1], lay, ref.config(layers=L, heads=H, bits_k=4, head_bits_v=tv)) == -5
    q = p.copy()
    q[ref.inspect(p)[4][4] + 3] = 7                      # a width that does not exist
    assert ref.decompress(q, out[0, 0], out[0, 1], lay, None) == -4
