"""Device self-test (run with -m gpu): the instruction sequences the quantizer kernels use in
place of IEEE division and subtraction give the IEEE result on every input of their domain."""
import pytest
import torch

from paper_2605_13734_amd import kvc

pytestmark = pytest.mark.gpu

NAMES = ["range/3", "range/7", "range/15", "range/255", "1/scale", "x-zero (packed fp16)", "float->byte"]


def test_arithmetic_shortcuts_are_exact():
    counts = torch.full((kvc.SELFTEST_COUNTS,), -1, dtype=torch.int64, device="cuda:0")
    rc = kvc.selftest(counts.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    got = counts.cpu().tolist()
    print("selftest mismatch counts:", dict(zip(NAMES, got)))
    assert got[:len(NAMES)] == [0] * len(NAMES), dict(zip(NAMES, got))
    assert got[len(NAMES):] == [0] * (kvc.SELFTEST_COUNTS - len(NAMES))
