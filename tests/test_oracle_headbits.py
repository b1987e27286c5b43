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


# ---- width tables together with the lossless stage ---------------------------------------------------
# Reading: chunks ordered by width (2, 3, 4, 8), then (layer, head, chunk); one code table per tensor
# and width, from a sample of that width's chunks; eight table slots, then the directory, then the
# width tables.  Pinned against uniform payloads of sub-tensors that hold one width's heads only.

TC = 128 * 3 + 41                    # several chunks per head and a ragged last one


@pytest.fixture(scope="module")
def long_data():
    return kvgen.as_u16(kvgen.make_kv(22, L, H, D, TC, torch.float16))


def heads_of(tab, b):
    return [lh for lh in range(L * H) if tab[lh] == b]


def test_lossless_stage_with_width_tables_round_trip_and_sizes(ref, long_data):
    tk, tv = tables(5)
    lay = ref.contiguous_layout(H, TC, D)
    plain = ref.config(layers=L, heads=H, head_bits_k=tk, head_bits_v=tv)
    coded = ref.config(layers=L, heads=H, head_bits_k=tk, head_bits_v=tv, codec=1)
    p0 = ref.compress(plain, long_data[0, 0], long_data[0, 1], lay, TC)
    p1 = ref.compress(coded, long_data[0, 0], long_data[0, 1], lay, TC)
    a, b = np.zeros_like(long_data), np.zeros_like(long_data)
    assert ref.decompress(p0, a[0, 0], a[0, 1], lay, plain) == 0
    assert ref.decompress(p1, b[0, 0], b[0, 1], lay, coded) == 0
    assert np.array_equal(a, b)                                   # the stage is lossless
    rc, _, tokens, total, sec = ref.inspect(p1)
    assert rc == 0 and tokens == TC and total == p1.size
    cph = -(-TC // 128)
    n = L * H * cph
    assert sec[5] == 8 * 256 + 4 * (2 * n + 1) + 2 * L * H         # eight tables, directory, two width tables
    d = p1[sec[4] + 2048: sec[4] + 2048 + 4 * (2 * n + 1)].view("<u4").astype(np.int64) * 16
    assert d[0] == 0 and np.all(np.diff(d) > 0)
    assert d[n] == sec[7] and d[2 * n] - d[n] == sec[9] and sec[8] == sec[6] + sec[7] and sec[6] + d[2 * n] == total
    assert np.array_equal(p1[sec[4] + 2048 + 4 * (2 * n + 1): sec[4] + 2048 + 4 * (2 * n + 1) + L * H], tk)
    assert np.array_equal(p1[sec[4] + 2048 + 4 * (2 * n + 1) + L * H: sec[4] + 2048 + 4 * (2 * n + 1) + 2 * L * H], tv)
    # metadata is that of the codec-free payload; the bound of kvc_payload_size holds
    assert np.array_equal(p1[sec[0]: sec[0] + sec[1]], p0[ref.inspect(p0)[4][0]: ref.inspect(p0)[4][0] + sec[1]])
    assert total <= ref.payload_size(coded, TC)[0]
    # every table slot is a complete prefix code or empty
    for is_v, tab in ((0, tk), (1, tv)):
        for wi, w in enumerate(WIDTHS):
            lens = p1[sec[4] + 256 * (4 * is_v + wi): sec[4] + 256 * (4 * is_v + wi + 1)].astype(np.int64)
            if heads_of(tab, w):
                assert lens.min() >= 1 and lens.max() <= 12 and (2 ** (12 - lens)).sum() == 2 ** 12
            else:
                assert not lens.any()


def test_every_width_is_coded_like_a_uniform_tensor_of_its_heads(ref, long_data):
    """The heads of one width, taken out into a tensor of their own (one layer, as many heads) and
    compressed with that uniform width and the lossless stage, give the table slot and, chunk after
    chunk, the bodies that the mixed payload holds for this width."""
    tk, tv = tables(6)
    lay = ref.contiguous_layout(H, TC, D)
    coded = ref.config(layers=L, heads=H, head_bits_k=tk, head_bits_v=tv, codec=1)
    p1 = ref.compress(coded, long_data[0, 0], long_data[0, 1], lay, TC)
    _, _, _, _, sec = ref.inspect(p1)
    cph = -(-TC // 128)
    n = L * H * cph
    d = p1[sec[4] + 2048: sec[4] + 2048 + 4 * (2 * n + 1)].view("<u4").astype(np.int64) * 16
    for is_v, tab in ((0, tk), (1, tv)):
        at = is_v * n                                             # directory index of the width's first chunk
        for wi, w in enumerate(WIDTHS):
            hs = heads_of(tab, w)
            if not hs:
                continue
            sub = np.zeros((1, 2, len(hs), TC, D), dtype=np.uint16)
            for i, lh in enumerate(hs):
                sub[0, :, i] = long_data[lh // H, :, lh % H]
            c = ref.config(layers=1, heads=len(hs), bits_k=w, bits_v=w, codec=1)
            q = ref.compress(c, sub[0, 0], sub[0, 1], ref.contiguous_layout(len(hs), TC, D), TC)
            _, _, _, _, s = ref.inspect(q)
            m = len(hs) * cph
            dq = q[s[4] + 512: s[4] + 512 + 4 * (2 * m + 1)].view("<u4").astype(np.int64) * 16
            assert np.array_equal(p1[sec[4] + 256 * (4 * is_v + wi): sec[4] + 256 * (4 * is_v + wi + 1)],
                                  q[s[4] + 256 * is_v: s[4] + 256 * (is_v + 1)]), ("table", is_v, w)
            sizes_mixed = np.diff(d[at: at + m + 1])
            sizes_sub = np.diff(dq[is_v * m: is_v * m + m + 1])
            assert np.array_equal(sizes_mixed, sizes_sub), ("sizes", is_v, w)
            got = p1[sec[6] + d[at]: sec[6] + d[at + m]]
            want = q[s[6] + dq[is_v * m]: s[6] + dq[is_v * m + m]]
            assert np.array_equal(got, want), ("bodies", is_v, w)
            at += m


def test_one_table_and_one_uniform_tensor_with_the_lossless_stage(ref, long_data):
    tk, _ = tables(7)
    lay = ref.contiguous_layout(H, TC, D)
    for kw in (dict(head_bits_k=tk, bits_v=4), dict(bits_k=3, head_bits_v=tk)):
        plain = ref.config(layers=L, heads=H, **kw)
        coded = ref.config(layers=L, heads=H, codec=1, **kw)
        a, b = np.zeros_like(long_data), np.zeros_like(long_data)
        assert ref.decompress(ref.compress(plain, long_data[0, 0], long_data[0, 1], lay, TC), a[0, 0], a[0, 1], lay, plain) == 0
        assert ref.decompress(ref.compress(coded, long_data[0, 0], long_data[0, 1], lay, TC), b[0, 0], b[0, 1], lay, coded) == 0
        assert np.array_equal(a, b)
