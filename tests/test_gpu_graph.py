"""GPU test (run with -m gpu): the calls of the library recorded into a HIP graph.  A graph is what
the allocation-free entry point is for; the library's own zero fills are kernels, not memsets, so a
replay must do what the eager call does.  Every replay is checked against the eager result, with eager
work and synchronisations between the replays and with new inputs in the same buffers."""
import numpy as np
import pytest
import torch

from paper_2605_13734_amd import kvc, kvgen

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("codec,static", [(kvc.CODEC_HUFF8, True), (kvc.CODEC_HUFF8, False), (kvc.CODEC_NONE, False)])
def test_graph_replays_match_eager_calls(ref, codec, static):
    L, H, T = 2, 4, 128 * 9 + 37
    plan = kvc.Plan(kvc.F16, L, H, 128, 4, 2, 32, 64, codec, max_tokens=T)
    x = kvgen.make_kv(60, L, H, 128, T, torch.float16, "cuda")
    y = torch.zeros_like(x)
    buf = kvc.Buffers(plan, [T])
    req_in, req_out = [kvc.contiguous_request(x, T)], [kvc.contiguous_request(y, T)]

    def run(stream):
        if static:
            kvc.compress_static(plan, req_in, buf.payload.data_ptr(), buf.offsets, buf.out_bytes.data_ptr(),
                                buf.status.data_ptr(), stream)
        else:
            buf.compress(req_in, stream)
        buf.decompress(req_out, stream)

    run(torch.cuda.current_stream().cuda_stream)         # eager once: set-up that a capture must not contain
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run(side.cuda_stream)
    cfg = ref.config(dtype=1, layers=L, heads=H, bits_k=4, bits_v=2, group_k=32, group_v=64, codec=codec)
    lay = ref.contiguous_layout(H, T, 128)
    for rep in range(4):
        x.copy_(kvgen.make_kv(61 + rep, L, H, 128, T, torch.float16, "cuda"))     # new input, same buffers
        buf.payload.fill_(0xCD)
        y.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert int(buf.status[0]) == 0
        got, out = buf.payload_of(0), y.cpu()
        # against the oracle (which also is what the eager path gives, by the parity tests)
        xu = kvgen.as_u16(x.cpu())
        want = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, T)
        assert np.array_equal(got, want), rep
        ru = np.zeros_like(xu)
        assert ref.decompress(want, ru[0, 0], ru[0, 1], lay, cfg) == 0
        assert np.array_equal(kvgen.as_u16(out), ru), rep
        # eager work between the replays
        run(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert np.array_equal(buf.payload_of(0), want)
