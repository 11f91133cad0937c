"""thia_op_nms_noalloc (the entry point for callers that cannot allocate device memory) against
thia_op_nms, through the C ABI: bit-exact keeps and counts on two calls in a row, the second
with a smaller input, so that whatever the first call left in the library's fixed buffer is
shown not to leak into the second."""
import numpy as np
import pytest
import torch

from gpu_common import MINI_FP32, gpu_model, to_dev

pytestmark = pytest.mark.gpu


def _rand_boxes(rs, n, size):
    x1 = rs.rand(n) * size
    y1 = rs.rand(n) * size
    w = 2 + rs.rand(n) * size / 3
    h = 2 + rs.rand(n) * size / 3
    return np.stack([x1, y1, x1 + w, y1 + h], 1).astype(np.float32)


def _case(rs, counts, cap, size):
    counts = np.asarray(counts, np.int32)
    boxes = np.zeros((len(counts), cap, 4), np.float32)
    for f, c in enumerate(counts):
        boxes[f, :c] = _rand_boxes(rs, c, size)
    return boxes, counts


def _both(m, boxes, counts, thr, max_keep):
    db, dc = to_dev(boxes), to_dev(counts)
    keep = torch.full((len(counts), max_keep), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((len(counts),), -7, dtype=torch.int32, device="cuda")
    m.op_nms_noalloc(db, dc, thr, max_keep, keep, cnt)
    torch.cuda.synchronize()
    ref_keep, ref_cnt = m.op_nms(db, dc, thr, max_keep)
    torch.cuda.synchronize()
    assert torch.equal(cnt, ref_cnt)
    assert torch.equal(keep, ref_keep)
    return cnt.cpu().numpy()


def test_nms_noalloc_matches_nms_on_two_calls_in_a_row():
    m, _ = gpu_model(MINI_FP32, 0xBEEF + 50)
    rs = np.random.RandomState(11)
    # first call: 8 frames at cap 2000 (250 000 of the buffer's 1 048 576 words), dense overlaps
    boxes, counts = _case(rs, [2000, 1937, 0, 1, 64, 65, 1999, 1024], 2000, 150.0)
    n1 = _both(m, boxes, counts, 0.7, 1000)
    assert n1[0] > 0 and n1[2] == 0 and n1[3] == 1
    # second call, smaller in every dimension: other boxes, other cap (other row pitch inside the buffer)
    boxes2, counts2 = _case(rs, [300, 77, 129], 300, 60.0)
    n2 = _both(m, boxes2, counts2, 0.5, 100)
    assert n2[0] > 0
    # and the first input again, after the small one
    assert np.array_equal(_both(m, boxes, counts, 0.7, 1000), n1)


def test_nms_noalloc_rejects_sizes_beyond_the_fixed_buffer():
    from paper_2102_08481_amd import ThiaError
    m, _ = gpu_model(MINI_FP32, 0xBEEF + 50)
    cap, n = 4096, 5                                       # 5 * 4096 * 64 words > 2^20
    boxes = torch.zeros((n, cap, 4), dtype=torch.float32, device="cuda")
    counts = torch.zeros((n,), dtype=torch.int32, device="cuda")
    keep = torch.full((n, 10), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(ThiaError) as e:
        m.op_nms_noalloc(boxes, counts, 0.7, 10, keep, cnt)
    assert e.value.code == -3
    torch.cuda.synchronize()
    assert int(keep.min()) == -7 and int(cnt.min()) == -7   # nothing was enqueued
    m.op_nms_noalloc(boxes[:4].contiguous(), counts[:4].contiguous(), 0.7, 10, keep[:4].contiguous(), cnt[:4].contiguous())
    torch.cuda.synchronize()
