"""esp_softmax_topk_static, the entry point that allocates nothing: its output against
esp_softmax_topk's on two calls in a row, the second with a smaller input (both share the one
device array of the library), through the C ABI.  The two run the same kernels, so ids and
probabilities must agree bit for bit; the oracle pins the first call as well."""
import numpy as np
import pytest
import torch

from util import O, synth, to_np

pytestmark = pytest.mark.gpu


def test_static_scratch_topk_matches_workspace_topk_on_two_calls():
    from paper_2603_17942_amd import binding as B
    B.load_library()
    assert torch.cuda.is_available(), "GPU tests need a GPU; there is no fallback path"
    cases = [(48, 128256, 10, 71), (3, 4096, 6, 72)]       # second call: fewer rows, fewer segments, smaller Kp
    inputs = []
    for rows, vocab, kp, seed in cases:                    # every buffer exists before the calls under test
        logits = synth.normal_like((rows, vocab), 2.0, seed, rows, "cuda", torch.float32)
        ids = torch.full((rows, kp), -5, dtype=torch.int32, device="cuda")
        ps = torch.full((rows, kp), -1.0, dtype=torch.float32, device="cuda")
        inputs.append((logits, kp, ids, ps))
    warm = torch.zeros((1, 64), dtype=torch.float32, device="cuda")
    B.softmax_topk(warm, 2)                                # the library's code object is resident before the measurement
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    for logits, kp, ids, ps in inputs:                     # two calls in a row, no synchronisation between them
        B.softmax_topk_static(logits, kp, ids, ps)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before     # nothing was allocated on the device
    for logits, kp, ids, ps in inputs:
        want_ids, want_ps = B.softmax_topk(logits, kp)
        assert torch.equal(ids, want_ids)
        assert torch.equal(ps, want_ps)
    logits, kp, ids, ps = inputs[0]
    lg = to_np(logits)
    for r in (0, 17, 47):
        o_ids, o_ps = O.softmax_topk(lg[r], kp)
        assert ids[r].tolist() == o_ids.tolist()
        np.testing.assert_allclose(ps[r].cpu().numpy(), o_ps, rtol=1e-4)
    # beyond the array: rejected with a clear error, outputs untouched
    rows, vocab, kp = 132, 128256, 32
    big = torch.zeros((rows, vocab), dtype=torch.float32, device="cuda")
    ids = torch.full((rows, kp), -5, dtype=torch.int32, device="cuda")
    ps = torch.full((rows, kp), -1.0, dtype=torch.float32, device="cuda")
    with pytest.raises(B.EspError) as ei:
        B.softmax_topk_static(big, kp, ids, ps)
    assert ei.value.code == 3                              # ESP_ECAPACITY
    torch.cuda.synchronize()
    assert int((ids != -5).sum()) == 0 and int((ps != -1.0).sum()) == 0
    # more rows fit when the vocabulary needs fewer segments
    small = synth.normal_like((300, 8192), 1.0, 73, 0, "cuda", torch.float32)
    ids = torch.empty((300, 4), dtype=torch.int32, device="cuda")
    ps = torch.empty((300, 4), dtype=torch.float32, device="cuda")
    B.softmax_topk_static(small, 4, ids, ps)
    w_ids, w_ps = B.softmax_topk(small, 4)
    assert torch.equal(ids, w_ids) and torch.equal(ps, w_ps)
