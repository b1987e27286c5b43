"""GPU test (run with -m gpu) of kvc_compress_static, the entry point for callers that cannot
allocate: its workspace is a static device array inside the library.  Called through the C ABI,
it must give the payload, size and status words of kvc_compress, byte for byte, on two calls in a
row that share the array, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvc, kvgen

pytestmark = pytest.mark.gpu


def both_ways(plan, x, T):
    st = torch.cuda.current_stream().cuda_stream
    req = [kvc.contiguous_request(x, T)]
    a = kvc.Buffers(plan, [T])
    a.payload.fill_(0xAB)
    a.compress(req, st)
    b = kvc.Buffers(plan, [T])
    b.payload.fill_(0xAB)
    b.out_bytes.fill_(-1)
    b.status.fill_(-1)
    kvc.compress_static(plan, req, b.payload.data_ptr(), b.offsets, b.out_bytes.data_ptr(), b.status.data_ptr(), st)
    torch.cuda.synchronize()
    assert int(a.status[0]) == 0 and int(b.status[0]) == 0
    assert int(a.out_bytes[0]) == int(b.out_bytes[0])
    assert np.array_equal(a.payload_of(0), b.payload_of(0))
    # and the payload it wrote decompresses
    y = torch.zeros_like(x)
    b.decompress([kvc.contiguous_request(y, T)], st)
    z = torch.zeros_like(x)
    a.decompress([kvc.contiguous_request(z, T)], st)
    torch.cuda.synchronize()
    assert int(b.status[0]) == 0
    assert torch.equal(y.view(torch.int16), z.view(torch.int16))
    return int(b.out_bytes[0])


def test_static_workspace_matches_caller_workspace():
    L, H = 3, 4
    x = kvgen.make_kv(77, L, H, 128, 128 * 21 + 9, torch.float16, "cuda")
    plan = kvc.Plan(kvc.F16, L, H, 128, 4, 4, 32, 32, kvc.CODEC_HUFF8, max_tokens=x.shape[3])
    assert 0 < plan.workspace_size() <= 4 << 20
    big = both_ways(plan, x, x.shape[3])                 # 264 chunks per tensor: several look-back windows
    small = both_ways(plan, x, 700)                      # the same array again, fewer chunks, ragged tail
    assert small < big
    both_ways(plan, x, x.shape[3])                       # and back up
    # without the coder nothing of the array is used; the call still has to match
    plain = kvc.Plan(kvc.F16, L, H, 128, 3, 8, 64, 32, kvc.CODEC_NONE, max_tokens=x.shape[3])
    both_ways(plain, x, 333)


def test_static_workspace_refuses_what_does_not_fit():
    huge = kvc.Plan(kvc.F16, 80, 8, 128, 4, 4, 32, 32, kvc.CODEC_HUFF8, max_tokens=1 << 20)
    assert huge.workspace_size() > 4 << 20
    x = kvgen.make_kv(78, 1, 1, 128, 32, torch.float16, "cuda")
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    out = torch.zeros(1, dtype=torch.int64, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(kvc.KvcError) as e:
        kvc.compress_static(huge, [kvc.contiguous_request(x, 32)], buf.data_ptr(), [0, 1 << 16], out.data_ptr(), status.data_ptr())
    assert e.value.status == -3                          # KVC_ERR_CAPACITY, before anything is launched
    tables = kvc.Plan(kvc.F16, 1, 1, 128, 0, 4, 32, 32, 0, max_tokens=32, head_bits_k=[2])
    with pytest.raises(kvc.KvcError) as e:
        kvc.compress_static(tables, [kvc.contiguous_request(x, 32)], buf.data_ptr(), [0, 1 << 16], out.data_ptr(), status.data_ptr())
    assert e.value.status == -2                          # KVC_ERR_UNSUPPORTED
