"""sk_top2_static, the entry point for callers that cannot allocate device memory (code under HIP
graph capture, tight serving loops): through the C ABI, against sk_top2 with a caller workspace,
bit for bit, on two calls in a row, the second with a smaller input (the fixed array inside the
library still holds the first call's pairs then), and its size limit."""
import ctypes

import pytest
import torch

import paper_2605_13784_amd as sk
from workloads import synth

pytestmark = pytest.mark.gpu


def _call_static(x, outs):
    idx1, idx2, val1, val2, gap = outs
    vp = ctypes.c_void_p
    rc = sk.lib().sk_top2_static(vp(x.data_ptr()), x.shape[0], x.shape[1], x.stride(0), vp(idx1.data_ptr()),
                                 vp(idx2.data_ptr()), vp(val1.data_ptr()), vp(val2.data_ptr()), vp(gap.data_ptr()),
                                 vp(torch.cuda.current_stream().cuda_stream))
    return rc


def test_static_scratch_entry_point_matches_the_workspace_one():
    gen = synth.generator(6, stream=9)
    L = sk.lib()
    # set-up call (rows == 0): resolves the array's device address, launches nothing
    assert L.sk_top2_static(None, 0, 128256, 128256, None, None, None, None, None, None) == sk.SK_OK
    for rows, vocab in ((48, 128256), (7, 33004)):            # the second call is the smaller one
        x = (2.5 * synth.draw(gen, (rows, vocab), "f32")).cuda()
        x[1, 5] = x[1, 900] = 40.0                               # a tie: lowest index first
        ref = sk.sk_top2(x)
        outs = sk.top2_outputs(rows, x.device)
        for t in outs:
            t.fill_(-1)
        assert _call_static(x, outs) == sk.SK_OK
        torch.cuda.synchronize()
        for got, want in zip(outs, ref):
            assert torch.equal(got, want)
        assert int(outs[0][1]) == 5 and int(outs[1][1]) == 900
    # beyond the fixed array: refused, outputs untouched
    rows = sk.SK_TOP2_STATIC_BYTES // 16 // 16 + 1                # 16 chunks of 8,192 logits per row, 16 bytes each
    x = torch.zeros((rows, 128256), dtype=torch.float32, device="cuda")
    outs = sk.top2_outputs(rows, x.device)
    outs[0].fill_(-7)
    assert _call_static(x, outs) == sk.SK_E_WORKSPACE
    torch.cuda.synchronize()
    assert int(outs[0][0]) == -7
    assert _call_static(x[:rows - 1], [t[:rows - 1] for t in outs]) == sk.SK_OK     # exactly at the limit
    torch.cuda.synchronize()
    assert int(outs[0][0]) == 0 and int(outs[1][0]) == 1
