"""GPU checks at sizes where every kernel runs well past its first batch of workgroups (run with
-m gpu).  The first 4 workgroups per CU start together on an idle chip; later ones start one at a
time beside workgroups that are in other phases of their work, and a mistake that needs that mix
does not show in small cases (the one that prompted this file: a 64-bit shift with its count in the
last allocated VGPR, which this GPU executes wrongly at three or four waves per SIMD, never showed in
the first 1024 workgroups).  For every code width, both tensor types and both strategy kinds:

* the lossless stage is exactly that: reconstructions with and without it are the same bits
  (a property that holds at any size), on three decompressions of the same payload;
* compressing twice gives the same payload bytes (the chunk-offset scan is order independent);
* sampled (layer, head) slices of the codec-free payload and reconstruction equal the oracle's.
"""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvc, kvgen
from test_gpu_full_size import check_sampled_heads

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
    if not kw:
        samples = [(0, 0, 0), (L - 1, 1, H - 1), (L // 2, 0, 3), (7, 1, 5)]
        check_sampled_heads(ref, plain, 0, lambda l, kv, h: x[l, kv, h].cpu(), lambda l, kv, h: y0[l, kv, h].cpu(),
                            L, H, T, dt, bits, bits, group, group, samples)
    del plain
    plan = kvc.Plan(dt, L, H, 128, bits, bits, group, group, 1, max_tokens=T, **kw)
    buf, y1 = run(plan, x)
    total = int(buf.out_bytes[0])
    first = buf.payload[:total].clone()
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
