"""GPU parity for per-head bit widths (run with -m gpu): payload bytes and reconstruction against
the oracle, contiguous and paged, with and without the rotation, batches, and the error paths."""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvc, kvgen

pytestmark = pytest.mark.gpu

WIDTHS = [2, 3, 4, 8]


def tables(seed, n):
    rng = np.random.default_rng(seed)
    return rng.choice(WIDTHS, n).astype(np.uint8), rng.choice(WIDTHS, n).astype(np.uint8)


def run(ref, x_cpu, tk, tv, gk, gv, transform=0, T=None, bits_k=4, bits_v=4, codec=0, anchor_period=0):
    L, _, H, Tfull, D = x_cpu.shape
    T = Tfull if T is None else T
    dt = 1 if x_cpu.dtype == torch.float16 else 2
    xu = kvgen.as_u16(x_cpu)
    cfg = ref.config(dtype=dt, layers=L, heads=H, bits_k=bits_k, bits_v=bits_v, group_k=gk, group_v=gv,
                     transform=transform, head_bits_k=tk, head_bits_v=tv, codec=codec, anchor_period=anchor_period)
    lay = ref.contiguous_layout(H, Tfull, D)
    want = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, T)
    x = x_cpu.cuda()
    plan = kvc.Plan(dt, L, H, D, bits_k, bits_v, gk, gv, codec, max_tokens=T, transform=transform,
                    head_bits_k=tk, head_bits_v=tv, anchor_period=anchor_period)
    assert plan.payload_size(T)[0] == ref.payload_size(cfg, T)[0]
    if not codec:
        assert plan.payload_size(T)[0] == want.size
    buf = kvc.Buffers(plan, [T])
    buf.payload.fill_(0xAB)
    st = torch.cuda.current_stream().cuda_stream
    buf.compress([kvc.contiguous_request(x, T)], st)
    torch.cuda.synchronize()
    assert int(buf.status[0]) == 0
    got = buf.payload_of(0)
    assert got.size == want.size, (got.size, want.size)
    d = np.nonzero(got != want)[0]
    assert d.size == 0, "first differing byte %d of %d (%d differ)" % (d[0], want.size, d.size)
    y = torch.full_like(x, 7.0)
    buf.decompress([kvc.contiguous_request(y, T)], st)
    torch.cuda.synchronize()
    assert int(buf.status[0]) == 0
    ru = np.zeros_like(xu)
    assert ref.decompress(want, ru[0, 0], ru[0, 1], lay, cfg) == 0
    assert np.array_equal(kvgen.as_u16(y.cpu())[:, :, :, :T], ru[:, :, :, :T])
    return buf, plan, want


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("group", [32, 64, 128])
def test_both_tables(ref, dtype, group):
    L, H = 3, 4
    x = kvgen.make_kv(80 + group, L, H, 128, 32 * 7 + 11, dtype)
    tk, tv = tables(group, L * H)
    run(ref, x, tk, tv, group, group)


def test_one_table_only_and_rotation(ref):
    L, H = 2, 8
    x = kvgen.make_kv(90, L, H, 128, 300, torch.float16)
    tk, tv = tables(7, L * H)
    run(ref, x, tk, None, 32, 32, bits_v=4)
    run(ref, x, None, tv, 64, 32, bits_k=2)
    run(ref, x, tk, tv, 32, 32, transform=1)
    run(ref, x, np.full(L * H, 8, np.uint8), np.full(L * H, 2, np.uint8), 32, 32, T=257)


def test_every_width_absent_but_one(ref):
    L, H = 1, 6
    x = kvgen.make_kv(91, L, H, 128, 100, torch.float16)
    for w in WIDTHS:
        run(ref, x, np.full(L * H, w, np.uint8), np.array([w, 2, w, 8, w, 3], np.uint8), 32, 32)


def test_paged_batch(ref):
    L, H, bt, P = 2, 2, 16, 40
    lens = [16 * 9 + 5, 77]
    tk, tv = tables(9, L * H)
    cfg = ref.config(dtype=1, layers=L, heads=H, group_k=32, group_v=32, head_bits_k=tk, head_bits_v=tv)
    plan = kvc.Plan(1, L, H, 128, 4, 4, 32, 32, 0, max_tokens=max(lens), max_batch=2, head_bits_k=tk, head_bits_v=tv)
    xs = [kvgen.make_kv(92 + i, L, H, 128, T, torch.float16) for i, T in enumerate(lens)]
    tabs = [kvgen.block_table(3 + i, -(-T // bt), P) for i, T in enumerate(lens)]
    pools = [kvgen.to_paged(x, t, bt, P).cuda() for x, t in zip(xs, tabs)]
    tabd = [t.cuda() for t in tabs]
    buf = kvc.Buffers(plan, lens)
    st = torch.cuda.current_stream().cuda_stream
    buf.compress([kvc.paged_request(p, t, T) for p, t, T in zip(pools, tabd, lens)], st)
    outs = [torch.zeros_like(p) for p in pools]
    buf.decompress([kvc.paged_request(o, t, T) for o, t, T in zip(outs, tabd, lens)], st)
    torch.cuda.synchronize()
    for i, T in enumerate(lens):
        assert int(buf.status[i]) == 0
        xu = kvgen.as_u16(xs[i])
        lay = ref.contiguous_layout(H, T, 128)
        want = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, T)
        assert np.array_equal(buf.payload_of(i), want)
        ru = np.zeros_like(xu)
        assert ref.decompress(want, ru[0, 0], ru[0, 1], lay, cfg) == 0
        assert np.array_equal(kvgen.as_u16(kvgen.from_paged(outs[i].cpu(), tabs[i], T)), ru)


def test_payload_of_another_table_is_refused(ref):
    L, H, T = 2, 4, 96
    x = kvgen.make_kv(93, L, H, 128, T, torch.float16)
    tk, tv = tables(10, L * H)
    buf, plan, want = run(ref, x, tk, tv, 32, 32)
    other = tk.copy()
    other[3] = 2 if tk[3] != 2 else 8                       # same sizes would be luck; usually differ
    plan2 = kvc.Plan(1, L, H, 128, 4, 4, 32, 32, 0, max_tokens=T, head_bits_k=other, head_bits_v=tv)
    buf2 = kvc.Buffers(plan2, [T])
    n = min(buf2.payload.numel(), want.size)
    buf2.payload[:n].copy_(torch.from_numpy(want[:n]).cuda())
    y = torch.zeros(L, 2, H, T, 128, dtype=torch.float16, device="cuda")
    buf2.decompress([kvc.contiguous_request(y, T)], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert int(buf2.status[0]) & 2                          # KVC_DEV_BAD_HEADER


def test_plan_rejections():
    with pytest.raises(kvc.KvcError):
        kvc.Plan(1, 1, 4, 128, 4, 4, 32, 32, 0, max_tokens=64, head_bits_k=[2, 3, 5, 8])


# ---- width tables together with the lossless stage: chunks by width, one code table per width ------------

@pytest.mark.parametrize("dtype,group", [(torch.float16, 32), (torch.bfloat16, 64), (torch.float16, 128)])
def test_both_tables_with_the_lossless_stage(ref, dtype, group):
    L, H, T = 3, 4, 128 * 4 + 37
    tk, tv = tables(11, L * H)
    x = kvgen.make_kv(31, L, H, 128, T, dtype)
    run(ref, x, tk, tv, group, group, codec=1)


def test_one_table_with_the_lossless_stage_transforms_and_short_requests(ref):
    L, H, T = 2, 4, 128 * 2 + 5
    tk, tv = tables(12, L * H)
    x = kvgen.make_kv(32, L, H, 128, T, torch.float16)
    run(ref, x, tk, None, 32, 64, bits_v=4, codec=1)
    run(ref, x, None, tv, 64, 32, bits_k=3, codec=1)
    run(ref, x, tk, tv, 32, 32, codec=1, transform=1)
    run(ref, x, tk, tv, 32, 32, codec=1, transform=2, anchor_period=32)
    run(ref, x, tk, tv, 32, 32, codec=1, T=1)
    only8 = np.full(L * H, 8, np.uint8)                       # one width only: seven empty table slots
    run(ref, x, only8, only8, 32, 32, codec=1)


def test_tables_with_the_lossless_stage_many_workgroups(ref):
    """Enough chunks per width that every width's launch spans many workgroups and look-back windows,
    in the dense fp16 layout that takes eight chunks per workgroup."""
    L, H, T = 8, 8, 128 * 24 + 3
    tk, tv = tables(13, L * H)
    x = kvgen.make_kv(33, L, H, 128, T, torch.float16)
    run(ref, x, tk, tv, 32, 32, codec=1)
