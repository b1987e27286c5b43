"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host
logic (plan validation, payload size, header inspection) agrees with the oracle's geometry.
No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2605_13734_amd import kvc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kvc.LIB_PATH):
        from paper_2605_13734_amd import build
        build.build()
    return kvc.load()


def test_exports_every_declared_symbol(lib):
    text = open(os.path.join(ROOT, "include", "kvc.h")).read()
    declared = set(re.findall(r"\b(kvc_[a-z_]+)\s*\(", text))
    assert declared == set(kvc.SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_plan_validation(lib):
    ok = dict(dtype=1, layers=2, kv_heads=2)
    kvc.Plan(**ok)
    bad = [dict(bits_k=5), dict(bits_v=0), dict(group_k=48), dict(group_v=16), dict(dtype=3),
           dict(layers=0), dict(codec=2), dict(max_batch=0), dict(max_tokens=-1),
           dict(transform=2), dict(transform=2, anchor_period=12), dict(transform=2, anchor_period=256),
           dict(transform=1, anchor_period=32)]
    for kw in bad:
        with pytest.raises(kvc.KvcError) as e:
            kvc.Plan(**{**ok, **kw})
        assert e.value.status == -1, kw
    unsupported = [dict(head_dim=64), dict(transform=3), dict(bits_k=16, codec=1)]
    for kw in unsupported:
        with pytest.raises(kvc.KvcError) as e:
            kvc.Plan(**{**ok, **kw})
        assert e.value.status == -2, kw
    assert kvc.status_string(-3) == "capacity too small"


@pytest.mark.parametrize("codec", [0, 1])
def test_payload_size_matches_oracle_geometry(lib, ref, codec):
    for (L, H, T, bk, bv, gk, gv) in [(1, 8, 1024, 4, 4, 32, 32), (32, 8, 8192, 2, 2, 64, 64),
                                      (3, 2, 1000, 4, 2, 64, 32), (1, 1, 1, 3, 3, 128, 128),
                                      (2, 4, 77, 8, 4, 32, 64), (1, 2, 0, 4, 4, 32, 32),
                                      (80, 8, 32768, 4, 4, 32, 32), (94, 4, 20001, 4, 2, 64, 64)]:
        plan = kvc.Plan(2, L, H, 128, bk, bv, gk, gv, codec, max_tokens=T)
        cfg = ref.config(dtype=2, layers=L, heads=H, bits_k=bk, bits_v=bv, group_k=gk, group_v=gv, codec=codec)
        assert plan.payload_size(T) == ref.payload_size(cfg, T)
        assert (plan.workspace_size() > 0) == bool(codec)
    if not codec:
        plan = kvc.Plan(1, 1, 1, 128, 2, 2, 32, 32, 0)
        n, exact = plan.payload_size(1 << 20)
        assert exact and abs(2 * (1 << 20) * 128 * 2 / n - 16 / 3) < 1e-3    # section 7.3: 5.33x


def test_sixteen_bit_sizes(lib, ref):
    plan = kvc.Plan(1, 2, 2, 128, 16, 4, 32, 64, 0)
    cfg = ref.config(layers=2, heads=2, bits_k=16, bits_v=4, group_k=32, group_v=64)
    assert plan.payload_size(77) == ref.payload_size(cfg, 77)


def test_inspect_reads_oracle_payloads(lib, ref):
    from paper_2605_13734_amd import kvgen
    x = kvgen.make_kv(0, 2, 2, 128, 150)
    xu = kvgen.as_u16(x)
    lay = ref.contiguous_layout(2, 150, 128)
    for codec in (0, 1):
        cfg = ref.config(layers=2, heads=2, bits_k=4, bits_v=3, group_k=64, group_v=32, codec=codec)
        p = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, 150)
        rc, m, s, tokens, total, sec = kvc.payload_inspect(p)
        assert rc == 0 and tokens == 150 and total == p.size
        assert (m.dtype, m.layers, m.kv_heads, m.head_dim) == (1, 2, 2, 128)
        assert (s.bits_k, s.bits_v, s.group_k, s.group_v, s.codec) == (4, 3, 64, 32, codec)
        assert sec == ref.inspect(p)[4]
        for pos, val in [(0, 0), (4, 9), (6, 7), (20, 5), (27, 1), (48, 1), (96, 3), (40, p[40] ^ 1)]:
            bad = p.copy()
            bad[pos] = val
            assert kvc.payload_inspect(bad)[0] == -4, pos
    bad = p.copy(); bad[16] = 64          # head_dim the kernels are not built for, otherwise well formed
    assert kvc.payload_inspect(bad)[0] in (-2, -4)


def test_block_table_check(lib):
    assert kvc.check_block_table([0, 5, 7], 8) == 0
    assert kvc.check_block_table([0, 8, 7], 8) == -1
    assert kvc.check_block_table([0, -1], 8) == -1


def test_host_errors_before_launch(lib):
    """Argument errors are returned without touching a device (there is none here)."""
    plan = kvc.Plan(1, 1, 1, max_tokens=64, max_batch=1)
    r = kvc.request(0x1000, 0x2000, 64, 128 * 64 * 2, 128 * 64, 128)
    with pytest.raises(kvc.KvcError) as e:
        kvc.compress(plan, [r], None, [0, 1 << 20], 0x100, 0x200)
    assert e.value.status == -1                                   # null payload
    with pytest.raises(kvc.KvcError) as e:
        kvc.compress(plan, [r], 0x10000, [0, 64], 0x100, 0x200)
    assert e.value.status == -3                                   # capacity
    with pytest.raises(kvc.KvcError) as e:
        kvc.compress(plan, [r, r], 0x10000, [0, 1 << 20, 2 << 20], 0x100, 0x200)
    assert e.value.status == -3                                   # batch larger than planned
    r2 = kvc.request(0x1000, 0x2000, 65, 128 * 64 * 2, 128 * 64, 128)
    with pytest.raises(kvc.KvcError) as e:
        kvc.compress(plan, [r2], 0x10000, [0, 1 << 20], 0x100, 0x200)
    assert e.value.status == -3                                   # more tokens than planned
    r3 = kvc.request(0x1004, 0x2000, 64, 128 * 64 * 2, 128 * 64, 128)
    with pytest.raises(kvc.KvcError) as e:
        kvc.compress(plan, [r3], 0x10000, [0, 1 << 20], 0x100, 0x200)
    assert e.value.status == -1                                   # misaligned tensor
    r4 = kvc.request(0x1000, 0x2000, 64, 0, 128, 256, 0x3000, 16 * 256, 12, 8)
    with pytest.raises(kvc.KvcError) as e:
        kvc.compress(plan, [r4], 0x10000, [0, 1 << 20], 0x100, 0x200)
    assert e.value.status == -2                                   # block size not a power of two


def test_newer_entry_points_refuse_on_the_host(lib):
    """kvc_stream_probe, kvc_workspace_init, kvc_table_bytes and kvc_compress_static: what the host can
    see is refused before a device is touched (there is none here)."""
    def status(fn, *a):
        with pytest.raises(kvc.KvcError) as e:
            fn(*a)
        return e.value.status

    assert status(kvc.stream_probe, 2, 0x1000, 0x2000, 128, 80) == -1       # no such mode
    assert status(kvc.stream_probe, 0, 0x1000, 0x2000, 100, 80) == -1       # rows not whole chunks
    assert status(kvc.stream_probe, 0, 0x1000, 0x2000, 128, 72) == -1       # payload rows not whole 16 bytes
    assert status(kvc.stream_probe, 1, 0x1000, 0x2000, 128, 272) == -1      # payload rows wider than the tensor's
    assert status(kvc.stream_probe, 0, 0x1004, 0x2000, 128, 80) == -1       # misaligned
    assert status(kvc.stream_probe, 0, None, 0x2000, 128, 80) == -1
    kvc.stream_probe(0, 0x1000, 0x2000, 0, 80)                              # nothing to do is not an error
    plain = kvc.Plan(1, 2, 2, max_tokens=64)
    assert lib.kvc_table_bytes(plain._h) == 0
    kvc.workspace_init(plain, None)                                         # no tables: nothing to bring over
    tk = np.array([2, 8, 4, 3], dtype=np.uint8)
    mixed = kvc.Plan(1, 2, 2, 128, 0, 4, 32, 32, 0, max_tokens=64, head_bits_k=tk)
    assert lib.kvc_table_bytes(mixed._h) > 0
    assert status(kvc.workspace_init, mixed, None) == -1                    # tables need a workspace
    assert status(kvc.workspace_init, mixed, 0x1004) == -1
    r = kvc.request(0x1000, 0x2000, 64, 128 * 64 * 2, 128 * 64, 128)
    assert status(kvc.compress_static, mixed, [r], 0x10000, [0, 1 << 20], 0x100, 0x200) == -2    # width tables
    huge = kvc.Plan(1, 80, 8, 128, 4, 4, 32, 32, 1, max_tokens=1 << 20)
    assert huge.workspace_size() > lib_static_bytes()
    assert status(kvc.compress_static, huge, [r], 0x10000, [0, 1 << 20], 0x100, 0x200) == -3    # larger than the static array


def lib_static_bytes():
    text = open(os.path.join(ROOT, "include", "kvc.h")).read()
    m = re.search(r"#define KVC_STATIC_WORKSPACE_BYTES \((\d+)u << (\d+)\)", text)
    return int(m.group(1)) << int(m.group(2))


def test_inspect_accepts_payloads_with_width_tables(ref):
    """kvc_payload_inspect on oracle payloads whose tensors carry per-head width tables."""
    import torch
    from paper_2605_13734_amd import kvgen
    L, H, T = 2, 3, 50
    x = kvgen.as_u16(kvgen.make_kv(1, L, H, 128, T, torch.float16))
    lay = ref.contiguous_layout(H, T, 128)
    tk = np.array([2, 3, 4, 8, 2, 8], np.uint8)
    for kw in (dict(head_bits_k=tk, bits_v=4), dict(bits_k=2, head_bits_v=tk), dict(head_bits_k=tk, head_bits_v=tk[::-1])):
        p = ref.compress(ref.config(layers=L, heads=H, **kw), x[0, 0], x[0, 1], lay, T)
        rc, model, strat, tokens, total, sec = kvc.payload_inspect(p[:128])
        assert rc == 0 and tokens == T and total == p.size
        assert (strat.bits_k == 0) == ("head_bits_k" in kw) and (strat.bits_v == 0) == ("head_bits_v" in kw)
        bad = p[:128].copy()
        bad[104] ^= 0x10                                   # K code bytes no longer match the offsets
        assert kvc.payload_inspect(bad)[0] != 0


def test_delta_transform_sizes_and_inspect(lib, ref):
    """Payload sizes with anchor rows against the oracle's geometry, and kvc_payload_inspect on
    oracle payloads of the delta transform."""
    import torch
    from paper_2605_13734_amd import kvgen
    for codec in (0, 1):
        for (L, H, T, bk, bv, period) in [(1, 8, 1024, 4, 4, 32), (3, 2, 1000, 4, 2, 32), (1, 1, 1, 3, 3, 128),
                                          (2, 4, 77, 8, 4, 64), (1, 2, 0, 4, 4, 64), (80, 8, 32768, 4, 4, 32)]:
            plan = kvc.Plan(2, L, H, 128, bk, bv, 32, 32, codec, max_tokens=T, transform=2, anchor_period=period)
            cfg = ref.config(dtype=2, layers=L, heads=H, bits_k=bk, bits_v=bv, codec=codec, transform=2, anchor_period=period)
            assert plan.payload_size(T) == ref.payload_size(cfg, T)
    plan = kvc.Plan(1, 2, 2, 128, 16, 4, 32, 32, 0, transform=2, anchor_period=32)      # K travels unchanged: V anchors only
    cfg = ref.config(layers=2, heads=2, bits_k=16, bits_v=4, transform=2, anchor_period=32)
    assert plan.payload_size(77) == ref.payload_size(cfg, 77)
    L, H, T = 2, 2, 150
    x = kvgen.as_u16(kvgen.make_kv(2, L, H, 128, T, torch.float16))
    lay = ref.contiguous_layout(H, T, 128)
    for codec in (0, 1):
        cfg = ref.config(layers=L, heads=H, codec=codec, transform=2, anchor_period=32)
        p = ref.compress(cfg, x[0, 0], x[0, 1], lay, T)
        rc, m, s, tokens, total, sec = kvc.payload_inspect(p)
        assert rc == 0 and tokens == T and total == p.size
        assert (s.transform, s.anchor_period) == (2, 32)
        assert sec == ref.inspect(p)[4]
        for pos, val in [(28, 64), (28, 0), (28, 33), (29, 1), (30, 1), (26, 1), (26, 3)]:
            bad = p.copy()
            bad[pos] = val
            assert kvc.payload_inspect(bad)[0] != 0, (pos, val)


def test_build_check_finds_a_shift_count_in_the_last_vgpr(tmp_path):
    """The build's assembly check: a 64-bit shift whose count is the last allocated VGPR is reported,
    the same instruction with a register allocated after the count, or a 32-bit shift, is not."""
    from paper_2605_13734_amd import build
    def asm(next_free, body):
        return ("\t.text\nkern:                                   ; @kern\n%s\ts_endpgm\n.Lfunc_end0:\n"
                "\t.amdhsa_kernel kern\n\t\t.amdhsa_group_segment_fixed_size 0\n\t\t.amdhsa_next_free_vgpr %d\n"
                "\t.end_amdhsa_kernel\n" % (body, next_free))
    cases = [(112, "\tv_lshlrev_b64 v[58:59], v111, v[26:27]\n", 1),
             (112, "\tv_lshrrev_b64 v[2:3], v111, v[4:5]\n\tv_ashrrev_i64 v[2:3], v111, v[4:5]\n", 2),
             (120, "\tv_lshlrev_b64 v[58:59], v111, v[26:27]\n", 0),       # v112.. are allocated
             (112, "\tv_lshlrev_b64 v[58:59], v109, v[26:27]\n", 0),       # not the last register
             (112, "\tv_lshlrev_b64 v[58:59], 9, v[110:111]\n", 0),        # constant count
             (112, "\tv_lshlrev_b32_e32 v5, v111, v4\n", 0),               # 32-bit shift
             (110, "\tv_lshlrev_b64 v[2:3], v103, v[4:5]\n", 0)]           # 8n+7, but registers follow it
    for i, (nf, body, want) in enumerate(cases):
        p = tmp_path / ("k%d.s" % i)
        p.write_text(asm(nf, body))
        hits = build.shift_count_in_last_vgpr(str(p))
        assert len(hits) == want, (i, hits)
        assert all(h[0] == "kern" for h in hits)


def test_inspect_never_accepts_a_damaged_header(lib, ref):
    """Every single-byte change of a valid header is either rejected by kvc_payload_inspect or
    leaves a header that the oracle also accepts with the same sections; without the lossless stage
    only the type and the transform can change that way (they do not enter the sizes)."""
    import torch
    from paper_2605_13734_amd import kvgen
    L, H, T = 2, 2, 150
    x = kvgen.as_u16(kvgen.make_kv(3, L, H, 128, T, torch.float16))
    lay = ref.contiguous_layout(H, T, 128)
    rng = np.random.default_rng(5)
    for kw in (dict(), dict(codec=1), dict(transform=1), dict(transform=2, anchor_period=64), dict(bits_k=16, bits_v=2, group_v=64)):
        p = ref.compress(ref.config(layers=L, heads=H, **kw), x[0, 0], x[0, 1], lay, T)
        assert kvc.payload_inspect(p)[0] == 0
        accepted = set()
        for pos in range(128):
            for val in {int(p[pos]) ^ 1, int(p[pos]) ^ 0x80, int(rng.integers(0, 256))} - {int(p[pos])}:
                bad = p.copy()
                bad[pos] = val
                rc, m, s, tokens, total, sec = kvc.payload_inspect(bad)
                if rc == 0:
                    accepted.add(pos)
                    orc, ocfg, otok, ototal, osec = ref.inspect(bad)
                    assert orc == 0 and otok == tokens and ototal == total and osec == sec, (kw, pos, val)
        # with the lossless stage the data-dependent sizes are only bounded, so a few more changes pass
        free = {6, 26} | ({22, 23} if kw.get("bits_k") == 16 else set())      # the group of a tensor stored unchanged is unused
        assert accepted <= free or kw.get("codec"), (kw, accepted)
    # a token count whose sizes wrap around 2^64 to those of a small one
    bad = p.copy()
    bad[39] = 4
    assert kvc.payload_inspect(bad)[0] == -4 and ref.inspect(bad)[0] == -4
