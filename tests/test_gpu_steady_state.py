"""GPU checks at sizes where every kernel runs well past its first batch of workgroups (run with
-m gpu).  The first 4 workgroups per CU start together on an idle chip; later ones start one at a
time beside workgroups that are in other phases of their work, and a mistake that needs that mix
does not show in small cases (the one that prompted this file: a 64-bit shift with its count in the
last allocated VGPR, which this GPU executes wrongly at three or four waves per SIMD, never showed in
the first 1024 workgroups).  For every code width, both tensor types and both strategy kinds:

* the lossless stage is exactly that: reconstructions with and without it are the same bits
  (a property that holds at any size), on three decompressions of the same payload;
* compressing twice gives the same payload bytes (the chunk-offset scan is order independent);
* sampled (layer, head) slices of the codec-free payload and reconstruction equal the oracle's,
  with and without a transform, and sampled coder bodies equal the oracle's byte for byte.
"""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvc, kvgen
from test_gpu_full_size import check_sampled_bodies, check_sampled_heads

pytestmark = pytest.mark.gpu

L, H, T = 24, 8, 8192              # 12288 chunks per section = 3072 (6144 at 8 bits) decode workgroups on 256 CUs


def run(plan, x, transform_note=""):
    buf = kvc.Buffers(plan, [T])
    st = torch.cuda.current_stream().cuda_stream
    buf.compress([kvc.contiguous_request(x)], st)
    y = torch.full_like(x, 7.0)
    buf.decompress([kvc.contiguous_request(y)], st)
    torch.cuda.synchronize()
    assert int(buf.status[0]) == 0, transform_note
    return buf, y


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("bits,group", [(2, 64), (3, 128), (4, 32), (8, 32), (4, 64)])
@pytest.mark.parametrize("kw", [dict(), dict(transform=1), dict(transform=2, anchor_period=32)], ids=["plain", "hadamard", "delta"])
def test_lossless_stage_changes_no_bit_far_past_the_first_batch(ref, dtype, bits, group, kw):
    dt = 1 if dtype == torch.float16 else 2
    x = kvgen.make_kv(90 + bits, L, H, 128, T, dtype, "cuda")
    st = torch.cuda.current_stream().cuda_stream
    plain, y0 = run(kvc.Plan(dt, L, H, 128, bits, bits, group, group, 0, max_tokens=T, **kw), x)
    samples = [(0, 0, 0), (L - 1, 1, H - 1), (L // 2, 0, 3), (7, 1, 5)]
    check_sampled_heads(ref, plain, 0, lambda l, kv, h: x[l, kv, h].cpu(), lambda l, kv, h: y0[l, kv, h].cpu(),
                        L, H, T, dt, bits, bits, group, group, samples, **kw)
    del plain
    plan = kvc.Plan(dt, L, H, 128, bits, bits, group, group, 1, max_tokens=T, **kw)
    buf, y1 = run(plan, x)
    total = int(buf.out_bytes[0])
    first = buf.payload[:total].clone()
    n = L * H * (T // 128)
    rng = np.random.default_rng(bits * 131 + group)
    picks = [(0, 0), (1, n - 1)] + [(int(rng.integers(0, 2)), int(rng.integers(0, n))) for _ in range(6)]
    check_sampled_bodies(ref, buf, lambda l, kv, h: x[l, kv, h].cpu(), L, H, T, dt, bits, bits, group, group, picks, **kw)
    for rep in range(3):
        bad = (y1.view(torch.int16) != y0.view(torch.int16))
        n = int(bad.sum())
        if n:
            where = bad.nonzero()[:4].tolist()
            raise AssertionError("%d elements differ from the codec-free reconstruction (decompression %d), first at %s" % (n, rep, where))
        y1.fill_(7.0)
        buf.decompress([kvc.contiguous_request(y1)], st)
        torch.cuda.synchronize()
        assert int(buf.status[0]) == 0
    buf.compress([kvc.contiguous_request(x)], st)
    torch.cuda.synchronize()
    assert int(buf.out_bytes[0]) == total
    assert torch.equal(buf.payload[:total], first)


def test_mixed_widths_and_groups_far_past_the_first_batch(ref):
    """K and V with different widths and groups (other kernel instantiations than the uniform cases)."""
    x = kvgen.make_kv(99, L, H, 128, T, torch.float16, "cuda")
    for bk, bv, gk, gv in ((4, 2, 64, 32), (8, 3, 128, 64), (2, 8, 32, 128)):
        _, y0 = run(kvc.Plan(1, L, H, 128, bk, bv, gk, gv, 0, max_tokens=T), x)
        _, y1 = run(kvc.Plan(1, L, H, 128, bk, bv, gk, gv, 1, max_tokens=T), x)
        assert torch.equal(y1.view(torch.int16), y0.view(torch.int16)), (bk, bv, gk, gv)


def test_per_head_widths_far_past_the_first_batch(ref):
    """Width tables (one launch per width over a head list) at the same size: sampled heads of every
    width against the oracle, codes, metadata and reconstruction."""
    rng = np.random.default_rng(7)
    tk = rng.choice([2, 3, 4, 8], L * H).astype(np.uint8)
    tv = rng.choice([2, 8], L * H).astype(np.uint8)
    x = kvgen.make_kv(98, L, H, 128, T, torch.float16, "cuda")
    plan = kvc.Plan(1, L, H, 128, 0, 0, 32, 32, 0, max_tokens=T, head_bits_k=tk, head_bits_v=tv)
    buf, y = run(plan, x)
    hdr = buf.payload[:128].cpu().numpy()
    rc, _, _, tokens, total, sec = kvc.payload_inspect(hdr)
    assert rc == 0 and tokens == T and total == int(buf.out_bytes[0])
    lay = ref.contiguous_layout(1, T, 128)
    picks = [(0, 0), (0, 1), (L * H - 1, 0), (L * H - 1, 1)]
    for w in (2, 3, 4, 8):                                   # one more head of every width
        picks.append((int(np.nonzero(tk == w)[0][len(np.nonzero(tk == w)[0]) // 2]), 0))
    for lh, kv in picks:
        table = tv if kv else tk
        bits = int(table[lh])
        l, h = divmod(lh, H)
        cfg1 = ref.config(dtype=1, layers=1, heads=1, bits_k=bits, bits_v=bits, group_k=32, group_v=32)
        xh = kvgen.as_u16(x[l, kv, h].cpu().contiguous())
        codes, meta = ref.compress_head(cfg1, kv, xh, lay, T, 0, 0)
        off = int(table[:lh].astype(np.int64).sum()) * T * 16          # widths of the heads before, 16 bytes per bit and row
        got = buf.payload[sec[8 if kv else 6] + off: sec[8 if kv else 6] + off + codes.size].cpu().numpy()
        assert np.array_equal(got, codes), ("codes", lh, kv, bits)
        mo = sec[2 if kv else 0] + lh * meta.size * 2
        got_meta = buf.payload[mo: mo + meta.size * 2].cpu().numpy().view(np.uint16)
        assert np.array_equal(got_meta, meta), ("meta", lh, kv, bits)
        back = np.zeros_like(xh)
        ref.decompress_head(cfg1, kv, codes, meta, T, 0, 0, back, lay)
        assert np.array_equal(kvgen.as_u16(y[l, kv, h].cpu().contiguous()), back), ("reconstruction", lh, kv, bits)
