"""moe_gate_topk_static, the entry point that allocates nothing (its arrival counters live in a device array of the
library), against moe_gate_topk on the same logits: bit-identical outputs on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from paper_2206_03382_amd import synth

pytestmark = pytest.mark.gpu


def test_gate_topk_static_matches_gate_topk():
    assert torch.cuda.is_available(), "this test needs a GPU"
    from paper_2206_03382_amd import moe
    L = moe.lib()
    limit = int(L.moe_gate_topk_static_max_bytes())
    assert limit == 8 << 20
    for T, E, k, f in ((20000, 128, 8, 2.0), (777, 12, 3, 0.5)):            # the second call is smaller than the first
        assert moe.gate_workspace_bytes(T, E, k) <= limit
        logits = synth.make_logits(T, E, seed=T + k, quantum=0.25)
        logits[:, 1] += 0.75                                                 # an overloaded expert: truncation at capacity
        C = moe.capacity(T, E, k, f)
        lg = torch.from_numpy(logits).cuda()
        ref = moe.gate_topk(lg, k, C, 1)
        out = dict(idx=torch.full((T, k), -7, dtype=torch.int32, device="cuda"), loc=torch.full((T, k), -7, dtype=torch.int32, device="cuda"),
                   gate_w=torch.full((T, k), float("nan"), device="cuda"), counts=torch.full((E,), -7, dtype=torch.int32, device="cuda"),
                   slot_src=torch.full((E, C), -7, dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        moe.gate_topk_static(lg, k, C, 1, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for key in ("idx", "loc", "counts", "slot_src"):
            assert torch.equal(out[key], ref[key]), (T, key)
        assert np.array_equal(out["gate_w"].cpu().numpy().view(np.uint32), ref["gate_w"].cpu().numpy().view(np.uint32))
    # beyond the static buffer: a clear error, nothing launched
    T, E, k = 1 << 20, 128, 8
    assert moe.gate_workspace_bytes(T, E, k) > limit
    fake = 4096
    assert L.moe_gate_topk_static(fake, T, E, k, 1024, 1, fake, fake, fake, fake, None, None) == moe.SCRATCH_TOO_SMALL
    assert b"static scratch" in L.moe_status_string(moe.SCRATCH_TOO_SMALL)
