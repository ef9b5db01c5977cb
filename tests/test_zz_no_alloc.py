"""samp_encoder_forward_noalloc (the entry point for callers that cannot allocate: its workspace is an array inside
the library's device image) against samp_encoder_forward: bit-identical outputs, on two calls in a row, the second
with a smaller input, so that whatever the first call left in the shared array is seen not to matter."""
import numpy as np
import pytest

import samp_workloads as W
from samp_workloads import FULL_INT8, FFN_INT8, MHA_INT8, FP16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2209_09130_amd as P
    P.lib()
    return P


def test_noalloc_forward_matches_forward_twice_in_a_row_second_call_smaller(P):
    import torch
    w = W.Workload("noalloc", 4, 256, 4, 512, 6, 72, (FULL_INT8, FFN_INT8, MHA_INT8, FP16), varlen=True, min_len=1,
                   plain_params=False, calib_batch=4, calib_seq=72)
    wts = W.make_weights(w)
    hid, lens, mask = W.make_hidden(w)
    cal = torch.from_numpy(W.make_calibration_batch(w)).cuda()
    a = (w.layers, w.hidden, w.heads, w.ffn, w.ln_eps)
    enc16 = P.Encoder(*a, (FP16,) * w.layers, wts, None, max_batch=w.batch, max_seq=w.seq)
    sc = enc16.calibrate(cal)
    enc16.close()
    enc = P.Encoder(*a, w.modes, wts, sc, max_batch=w.batch, max_seq=w.seq)
    enc.set_graph(False)
    enc.set_groups(1)
    for (B, S, use_mask) in ((6, 72, True), (3, 40, True), (2, 16, False)):
        h = torch.from_numpy(np.ascontiguousarray(hid[:B, :S])).cuda()
        m = torch.from_numpy(np.ascontiguousarray(np.minimum(mask[:B, :S], 1))).cuda() if use_mask else None
        if m is not None:
            m[:, 0] = 1                                           # every sequence keeps at least one token
        want = enc.forward(h, m, torch.full_like(h, 3.0)).clone()
        torch.cuda.synchronize()
        got = enc.forward_noalloc(h, m, torch.full_like(h, -5.0))
        torch.cuda.synchronize()
        assert torch.equal(got, want), (B, S)
    # a batch whose workspace does not fit the built-in array is refused with a message, nothing is launched
    big = P.Encoder(*a, w.modes, wts, sc, max_batch=64, max_seq=512)
    hb = torch.zeros((64, 512, w.hidden), dtype=torch.float16, device="cuda")
    with pytest.raises(P.SampError) as e:
        big.forward_noalloc(hb, None, torch.empty_like(hb))
    assert e.value.code == -3 and "scratch" in str(e.value)
    big.close()
    enc.close()
