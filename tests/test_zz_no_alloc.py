"""The entry point that allocates nothing (rf_arm_classify_noalloc, for callers that cannot call
hipMalloc or carry a workspace) against rf_arm_classify: same kernels on the library's static
scratch, so classes and recalls must be identical; two calls in a row, the second on a smaller
input, so that whatever the first call left in the scratch is seen not to matter."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2505_21036_amd as rf
import rf_inputs as inp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def one_call(name, mode, alpha, scale):
    w = inp.WORKLOADS[name]
    print("case no-alloc", name, mode, alpha, flush=True)
    rl, ol = rf.rf_layout(w.T, w.H, w.W, w.text_len), orc.Layout(w.T, w.H, w.W, w.text_len)
    Q, K, _ = inp.full_qkv(w, DEV, scale)
    hc = torch.full((w.B, w.nH), -5, dtype=torch.int32, device=DEV)
    rec = torch.full((w.B, w.nH, 2), -1.0, dtype=torch.float32, device=DEV)
    assert rf.rf_arm_workspace_bytes(w.B, w.nH, rl) <= rf.RF_ARM_STATIC_SCRATCH_BYTES
    before = torch.cuda.memory_allocated()
    rf.rf_arm_classify_noalloc(Q, K, rl, None, mode, alpha, hc, rec)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before  # nothing of torch's was allocated on the way
    hc_ref, rec_ref = rf.rf_arm_classify(Q, K, rl, None, mode, alpha)
    torch.cuda.synchronize()
    assert torch.equal(hc, hc_ref) and torch.equal(rec, rec_ref), (hc, hc_ref, rec, rec_ref)
    # and both against the oracle, to the bar of the other ARM tests
    hc_h, rec_h = hc.cpu().numpy(), rec.cpu().numpy()
    for b in range(w.B):
        for h in range(w.nH):
            q, k, _ = (t.float().numpy() for t in inp.head_qkv(w, b, h, scale))
            c, (rh, rt) = orc.arm_classify(q, k, ol, orc.Params(), mode, alpha)
            assert abs(rec_h[b, h, 0] - rh) <= 1e-3 and abs(rec_h[b, h, 1] - rt) <= 1e-3, (b, h, rec_h[b, h], rh, rt)
            decided_by_near = (abs(rh - alpha) < 1e-3) or (rh < alpha and abs(rt - alpha) < 1e-3)
            if decided_by_near:
                print("head", (b, h), "within 1e-3 of the threshold (exempt):", rh, rt, flush=True)
            else:
                assert hc_h[b, h] == c, (b, h, hc_h[b, h], c, rh, rt)


def test_noalloc_matches_the_workspace_entry_point_twice_in_a_row():
    one_call("ragged128", rf.RF_SAMPLE_FIRST_FRAME, 0.45, 3.0)      # 6 heads, 130 + 130 sampled rows
    one_call("tiny", rf.RF_SAMPLE_EQUAL_INTERVAL, 0.5, 1.0)         # smaller: 2 heads, 64 rows
    one_call("ragged96", rf.RF_SAMPLE_EQUAL_INTERVAL, 0.3, 2.0)


def test_noalloc_refuses_what_does_not_fit():
    rl = rf.rf_layout(33, 45, 80, 256)
    w = inp.WORKLOADS["tiny"]
    Q, K, _ = inp.full_qkv(w, DEV)
    hc = torch.empty(25, 3, dtype=torch.int32, device=DEV)
    rec = torch.empty(25, 3, 2, dtype=torch.float32, device=DEV)
    lib = rf.load_library()
    import ctypes as C
    st = lib.rf_arm_classify_noalloc(Q.data_ptr(), K.data_ptr(), 25, 3, 64, C.byref(rl), None, 0, 0.9, hc.data_ptr(),
                                     rec.data_ptr(), None)
    assert st == -6 and "workspace" in rf.rf_status_string(st)
