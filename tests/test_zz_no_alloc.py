"""flover_k_decode_attention_noalloc (the entry point for callers that cannot allocate) against
flover_k_decode_attention on the same inputs, through the C ABI: same kernels, so the outputs must be equal bit for
bit; two calls in a row on the library's one scratch array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import flover_synth as synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fl():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2305_13484_amd as m
    m.load_library()
    return m


@pytest.mark.parametrize("dtype,d", [(synth.DT_BF16, 128), (synth.DT_F16, 64), (synth.DT_F32, 128)])
def test_noalloc_attention_equals_the_workspace_entry_point_twice_in_a_row(fl, dtype, d):
    print("noalloc attention", dtype, d, flush=True)
    Cn, nh, S = 40, 8, 700
    # first call: 37 rows, lengths across the 256-position chunk boundaries; second call: 5 rows, short
    for M, lo, hi, seed in ((37, 1, S, 5), (5, 1, 90, 6)):
        q, k, v, slots, lens = synth.attention_case(seed + d, M, Cn, nh, d, S, dtype, lo, hi)
        if M > 6:
            lens[:6] = [1, 2, 255, 256, 257, S]
        qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
        ref = fl.k_decode_attention(qd, kd, vd, slots, lens)
        out = torch.full_like(ref, float("nan"))
        got = fl.k_decode_attention_noalloc(qd, kd, vd, slots, lens, out)
        torch.cuda.synchronize()
        assert torch.isfinite(got.float()).all()
        assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), (M, dtype, d)


def test_noalloc_attention_limits_and_bad_arguments(fl):
    dtype, d, nh = synth.DT_BF16, 128, 32
    # more rows than one call serves
    q, k, v, slots, lens = synth.attention_case(1, 257, 4, 4, 64, 16, dtype, 1, 16)
    slots = np.arange(257, dtype=np.int32) % 4
    out = torch.empty_like(q, device="cuda")
    with pytest.raises(fl.FloverError, match="at most 256 rows"):
        fl.k_decode_attention_noalloc(q.cuda(), k.cuda(), v.cuda(), slots, lens, out)
    # a workspace beyond the built-in scratch: 256 rows x 16 chunks x 32 heads x (128 + 2) floats = 68 MB
    S, M = 4096, 256
    q = torch.zeros((M, nh, d), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((1, nh, S, d), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fl.FloverError, match="exceeds the built-in scratch"):
        fl.k_decode_attention_noalloc(q, kv, kv, np.zeros(M, np.int32), np.full(M, S, np.int32), torch.empty_like(q))
    # the same checks as the workspace entry point
    q, k, v, slots, lens = synth.attention_case(1, 2, 3, 4, 64, 32, dtype, 1, 32)
    bad = lens.copy()
    bad[0] = 33
    with pytest.raises(fl.FloverError):
        fl.k_decode_attention_noalloc(q.cuda(), k.cuda(), v.cuda(), slots, bad, torch.empty_like(q, device="cuda"))
    out = fl.k_decode_attention_noalloc(q.cuda()[:0].contiguous(), k.cuda(), v.cuda(), slots[:0], lens[:0],
                                        torch.empty_like(q[:0], device="cuda"))
    assert out.shape[0] == 0
    # and it still works after the refused calls
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    ref = fl.k_decode_attention(qd, kd, vd, slots, lens)
    got = fl.k_decode_attention_noalloc(qd, kd, vd, slots, lens, torch.empty_like(ref))
    assert torch.equal(got, ref)
