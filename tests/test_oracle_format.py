"""Pins for the oracle's packing, payload geometry, layouts and whole-request round trip."""
import os

import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvgen
from util import bits_to_f64, f16_bits_to_f64, unpack_int, unpack_np

GOLD = os.path.join(os.path.dirname(__file__), "golden")
BITS = [2, 3, 4, 8]


def golden(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].strip()
        if "=" in line and not line.startswith("b"):
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


# ---- packing -------------------------------------------------------------------------------

def test_pack_hand_written_rows(ref):
    n = 0
    for line in open(os.path.join(GOLD, "pack_rows.txt")):
        line = line.split("#")[0].strip()
        if not line.startswith("b"):
            continue
        b, codes, by = line.split()
        bits = int(b[1:])
        codes = np.array([int(c) for c in codes.split("=")[1].split(",")], dtype=np.uint8)
        want = bytes.fromhex(by.split("=")[1])
        assert bytes(ref.pack(codes, bits)) == want
        assert np.array_equal(ref.unpack(np.frombuffer(want, dtype=np.uint8), codes.size, bits), codes)
        n += 1
    assert n == 5


@pytest.mark.parametrize("bits", BITS)
def test_pack_exhaustive_value_by_position(ref, bits):
    """Every code value at every one of 8 positions, others zero / all ones; the expected bytes
    come from one big Python integer (sum of q_i << i*b), not from a bit loop."""
    top = (1 << bits) - 1
    for fill in (0, top):
        for pos in range(8):
            for val in range(top + 1):
                q = np.full(8, fill, dtype=np.uint8)
                q[pos] = val
                big = sum(int(q[i]) << (i * bits) for i in range(8))
                want = big.to_bytes(bits, "little")
                got = ref.pack(q, bits)
                assert bytes(got) == want
                assert np.array_equal(ref.unpack(got, 8, bits), q)


@pytest.mark.parametrize("bits", BITS)
def test_pack_random_against_big_integer(ref, bits):
    rng = np.random.default_rng(bits)
    q = rng.integers(0, 1 << bits, 1024).astype(np.uint8)
    got = ref.pack(q, bits)
    assert got.size == 1024 * bits // 8
    assert np.array_equal(unpack_int(got, 1024, bits), q)
    assert np.array_equal(unpack_np(got, bits), q)


# ---- payload size --------------------------------------------------------------------------

def closed_form(L, H, D, T, bk, bv, gk, gv):
    a16 = lambda n: (n + 15) // 16 * 16
    mk = 0 if bk == 16 else 4 * L * H * (-(-T // gk)) * D
    mv = 0 if bv == 16 else 4 * L * H * T * (D // gv)
    return 128 + a16(mk) + a16(mv) + a16(L * H * T * D * bk // 8) + a16(L * H * T * D * bv // 8)


def test_payload_size_paper_limit(ref):
    """Section 7.3: 2-bit, group-32 quantization of 16-bit KV cannot exceed about 5.33x because
    of its per-group metadata; without metadata it would be 8x."""
    gold = golden("paper_values.txt")
    T = 1 << 20
    cfg = ref.config(layers=1, heads=1, bits_k=2, bits_v=2, group_k=32, group_v=32)
    n, exact = ref.payload_size(cfg, T)
    cr = (2 * T * 128 * 2) / n
    assert exact and abs(cr - 16 / 3) < 1e-3 and round(cr, 2) == gold["cr_limit_2bit_group32"]
    assert 16 / 2 == gold["cr_ideal_2bit"]
    for b in BITS:
        for g in (32, 64, 128):
            cfg = ref.config(layers=2, heads=2, bits_k=b, bits_v=b, group_k=g, group_v=g)
            n, _ = ref.payload_size(cfg, T)
            assert abs((2 * 2 * 2 * T * 128 * 2) / n - 16 / (b + 32 / g)) < 1e-3


def test_payload_size_configs(ref):
    """Closed forms of the benchmark configurations."""
    cfg = ref.config(layers=1, heads=8, bits_k=4, bits_v=4)
    assert ref.payload_size(cfg, 1024)[0] == 1310848 == closed_form(1, 8, 128, 1024, 4, 4, 32, 32)
    cfg = ref.config(dtype=2, layers=32, heads=8, bits_k=2, bits_v=2, group_k=64, group_v=64)
    assert ref.payload_size(cfg, 8192)[0] == 167772288
    cfg = ref.config(dtype=2, layers=32, heads=8, bits_k=4, bits_v=4)
    assert ref.payload_size(cfg, 8192)[0] == 335544448
    # mixed K4 / V2 at group 64: 3.5 bits per element
    cfg = ref.config(dtype=2, layers=94, heads=4, bits_k=4, bits_v=2, group_k=64, group_v=64)
    T = 16384
    n, _ = ref.payload_size(cfg, T)
    assert n - 128 == 94 * 4 * T * 128 * 2 * 3.5 / 8
    # ragged tail, odd sizes, pass-through
    for (L, H, T, bk, bv, gk, gv) in [(3, 2, 1000, 4, 2, 64, 32), (1, 1, 1, 3, 3, 128, 128),
                                      (2, 4, 77, 16, 4, 32, 64), (1, 2, 0, 4, 4, 32, 32),
                                      (2, 1, 129, 8, 16, 128, 32)]:
        cfg = ref.config(layers=L, heads=H, bits_k=bk, bits_v=bv, group_k=gk, group_v=gv)
        assert ref.payload_size(cfg, T)[0] == closed_form(L, H, 128, T, bk, bv, gk, gv)


def test_llama70b_kv_volume():
    """Section 1 quotes 39.06 GB of KV for Llama-3.1-70B at 128K tokens: 80 layers, 8 KV heads,
    head_dim 128, K and V, 2 bytes -- the shape the 70B benchmark config uses."""
    gold = golden("paper_values.txt")
    per_token = 80 * 8 * 128 * 2 * 2
    assert round(per_token * 128000 / 2 ** 30, 2) == gold["llama70b_kv_gib_128k"]


def test_config_errors(ref):
    bad = [dict(bits_k=5), dict(bits_v=1), dict(group_k=48), dict(group_v=48), dict(head_dim=100),
           dict(dtype=3), dict(layers=0), dict(group_k=256), dict(codec=2)]
    for kw in bad:
        with pytest.raises(ValueError):
            ref.payload_size(ref.config(**kw), 16)
    with pytest.raises(ValueError):
        ref.payload_size(ref.config(bits_k=16, codec=1), 16)
    with pytest.raises(ValueError):
        ref.payload_size(ref.config(), -1)


# ---- whole request -------------------------------------------------------------------------

def tiny(seed, L, H, T, dtype=torch.float16):
    x = kvgen.make_kv(seed, L, H, 128, T, dtype, "cpu")
    return x, kvgen.as_u16(x)


def run(ref, cfg, xu, T):
    lay = ref.contiguous_layout(cfg.heads, T, cfg.head_dim)
    return ref.compress(cfg, xu[0, 0], xu[0, 1], lay, T), lay


@pytest.mark.parametrize("bits,group", [(2, 64), (3, 32), (4, 32), (8, 128)])
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_round_trip_error_bound(ref, bits, group, dtype):
    L, H, T = 2, 2, 200                     # ragged K tail: 200 = 3*64 + 8 = 6*32 + 8 = 128 + 72
    dt = 1 if dtype == torch.float16 else 2
    x, xu = tiny(3, L, H, T, dtype)
    cfg = ref.config(dtype=dt, layers=L, heads=H, bits_k=bits, bits_v=bits, group_k=group, group_v=group)
    payload, lay = run(ref, cfg, xu, T)
    assert payload.size == ref.payload_size(cfg, T)[0]
    out = np.zeros_like(xu)
    assert ref.decompress(payload, out[0, 0], out[0, 1], lay, cfg) == 0
    x64 = bits_to_f64(xu, dt)
    y64 = bits_to_f64(out, dt)
    # per group: |x - x^| <= scale/2 + half an output ulp (+ scale rounding at the top level)
    qmax = (1 << bits) - 1
    half_ulp = np.abs(y64) * (2.0 ** -11 if dt == 1 else 2.0 ** -8)
    for kv in range(2):
        xs, ys = x64[:, kv], y64[:, kv]
        if kv == 0:
            pad = (-T) % group
            xp = np.pad(xs, ((0, 0), (0, 0), (0, pad), (0, 0)), mode="edge")
            g = xp.reshape(L, H, -1, group, 128)
            rng_ = np.repeat(g.max(axis=3) - g.min(axis=3), group, axis=2)[:, :, :T]
        else:
            g = xs.reshape(L, H, T, 128 // group, group)
            rng_ = np.repeat(g.max(axis=4) - g.min(axis=4), group, axis=3)
        step = rng_ / qmax
        assert np.all(np.abs(xs - ys) <= step * (0.5 + qmax * 2.0 ** -11 + 2.0 ** -10) + half_ulp[:, kv] + 1e-12)


def test_header_and_sections(ref):
    L, H, T = 2, 3, 100
    x, xu = tiny(4, L, H, T)
    cfg = ref.config(layers=L, heads=H, bits_k=4, bits_v=2, group_k=64, group_v=32)
    payload, lay = run(ref, cfg, xu, T)
    rc, c2, tokens, total, sec = ref.inspect(payload)
    assert rc == 0 and tokens == T and total == payload.size
    assert bytes(payload[:4]) == b"KVC1" and payload[4] == 1 and payload[5] == 0
    for f in ("dtype", "layers", "heads", "head_dim", "bits_k", "bits_v", "group_k", "group_v", "codec"):
        assert getattr(c2, f) == getattr(cfg, f)
    mk, mv = 4 * L * H * 2 * 128, 4 * L * H * T * 4
    ck, cv = L * H * T * 128 * 4 // 8, L * H * T * 128 * 2 // 8
    assert sec == [128, mk, 128 + mk, mv, 128 + mk + mv, 0, 128 + mk + mv, ck, 128 + mk + mv + ck, cv]
    # sections hold what the per-head entry point produces, heads in [l][h] order
    for l in range(L):
        for h in range(H):
            lh = l * H + h
            ck_, mk_ = ref.compress_head(cfg, 0, xu[0, 0], lay, T, l, h)
            cv_, mv_ = ref.compress_head(cfg, 1, xu[0, 1], lay, T, l, h)
            assert np.array_equal(payload[sec[6] + lh * ck_.size: sec[6] + (lh + 1) * ck_.size], ck_)
            assert np.array_equal(payload[sec[8] + lh * cv_.size: sec[8] + (lh + 1) * cv_.size], cv_)
            assert np.array_equal(payload[sec[0] + lh * mk_.size * 2: sec[0] + (lh + 1) * mk_.size * 2].view(np.uint16), mk_)
            assert np.array_equal(payload[sec[2] + lh * mv_.size * 2: sec[2] + (lh + 1) * mv_.size * 2].view(np.uint16), mv_)
    # corrupt headers are rejected
    bad = payload.copy(); bad[0] = ord("X")
    assert ref.decompress(bad, xu[0, 0].copy(), xu[0, 1].copy(), lay) != 0
    bad = payload.copy(); bad[20] = 5
    assert ref.decompress(bad, xu[0, 0].copy(), xu[0, 1].copy(), lay) != 0
    assert ref.decompress(payload[:-16], xu[0, 0].copy(), xu[0, 1].copy(), lay) != 0
    other = ref.config(layers=L, heads=H, bits_k=4, bits_v=4, group_k=64, group_v=32)
    assert ref.decompress(payload, xu[0, 0].copy(), xu[0, 1].copy(), lay, other) != 0


def test_sixteen_bits_is_identity(ref):
    """The bypass profile (section 7.2: KVServe skips compression when it would not pay)."""
    L, H, T = 2, 2, 37
    for dtype, dt in ((torch.float16, 1), (torch.bfloat16, 2)):
        x, xu = tiny(5, L, H, T, dtype)
        cfg = ref.config(dtype=dt, layers=L, heads=H, bits_k=16, bits_v=16)
        payload, lay = run(ref, cfg, xu, T)
        assert payload.size == 128 + xu.size * 2
        assert np.array_equal(payload[128:128 + xu.size].view(np.uint16).reshape(L, H, T, 128), xu[:, 0])
        out = np.zeros_like(xu)
        assert ref.decompress(payload, out[0, 0], out[0, 1], lay, cfg) == 0
        assert np.array_equal(out, xu)


def test_ragged_tail_group_is_standalone(ref):
    """T = 2*32 + 5: the last K group spans 5 tokens and equals a 5-token request's only group."""
    H, T = 1, 69
    x, xu = tiny(6, 1, H, T)
    cfg = ref.config(heads=H, bits_k=4, group_k=32)
    lay = ref.contiguous_layout(H, T, 128)
    codes, meta = ref.compress_head(cfg, 0, xu[0, 0], lay, T, 0, 0)
    tail = np.ascontiguousarray(xu[0, 0, 0, 64:])
    lay5 = ref.contiguous_layout(H, 5, 128)
    c5, m5 = ref.compress_head(cfg, 0, tail, lay5, 5, 0, 0)
    assert np.array_equal(codes[64 * 64:], c5)
    assert np.array_equal(meta[2 * 2 * 128:], m5)


@pytest.mark.parametrize("codec", [0, 1])
def test_paged_equals_contiguous(ref, codec):
    """Any block-table permutation gives the payload of the same logical data stored
    contiguously; decompressing into a different permutation and gathering gives the
    contiguous decompression."""
    L, H, T, bt = 2, 2, 16 * 9 + 5, 16
    x, xu = tiny(7, L, H, T)
    cfg = ref.config(layers=L, heads=H, bits_k=4, bits_v=3, group_k=64, group_v=32, codec=codec)
    want, lay = run(ref, cfg, xu, T)
    nb, P = -(-T // bt), 16
    tab = kvgen.block_table(1, nb, P)
    pool = kvgen.to_paged(x, tab, bt, P)
    pu = kvgen.as_u16(pool)
    play = ref.paged_layout(H, 128, bt, P, tab.numpy())
    got = ref.compress(cfg, pu[0, 0], pu[0, 1], play, T)
    assert np.array_equal(got, want)
    tab2 = kvgen.block_table(2, nb, P)
    out_pool = torch.zeros_like(pool)
    ou = kvgen.as_u16(out_pool)
    play2 = ref.paged_layout(H, 128, bt, P, tab2.numpy())
    assert ref.decompress(got, ou[0, 0], ou[0, 1], play2, cfg) == 0
    flat = np.zeros_like(xu)
    assert ref.decompress(want, flat[0, 0], flat[0, 1], lay, cfg) == 0
    gathered = kvgen.as_u16(kvgen.from_paged(out_pool, tab2, T))
    assert np.array_equal(gathered, flat)


def test_generator_recipe():
    """Input recipe: V ~ N(0,1); K channels log-normally scaled with 4 outlier channels x20."""
    x = kvgen.make_kv(0, 1, 8, 128, 1024).float()
    v = x[0, 1]
    assert abs(float(v.mean())) < 0.01 and abs(float(v.std()) - 1) < 0.01
    s = kvgen.channel_scales(0, 1, 8, 128)
    kstd = x[0, 0].std(dim=1)                     # [H, D]
    assert torch.allclose(kstd, s[0], rtol=0.15)
    gains = torch.sort(s[0] / torch.exp(torch.log(s[0]).median()), dim=-1).values
    assert (s[0] > 0).all()
    again = kvgen.make_kv(0, 1, 8, 128, 1024)
    assert torch.equal(again, kvgen.make_kv(0, 1, 8, 128, 1024))
    assert not torch.equal(again, kvgen.make_kv(1, 1, 8, 128, 1024))
    # counter-based: an element depends on its coordinates and the seed alone
    assert torch.equal(kvgen.make_kv(0, 1, 8, 128, 300), again[:, :, :, :300])
    two = kvgen.make_kv(0, 2, 8, 128, 64)
    assert torch.equal(two[0], again[0, :, :, :64]) and not torch.equal(two[1], two[0])
    tab = kvgen.block_table(3, 64, 64)
    assert sorted(tab.tolist()) == list(range(64))
    lens = kvgen.request_lengths(0, 4, 16384, 32768)
    assert all(16384 <= n <= 32768 for n in lens) and lens == kvgen.request_lengths(0, 4, 16384, 32768)
