"""skvq_decode_attention_static (the entry point that allocates nothing; its split partials live in
a fixed array of the library's device image) against skvq_decode_attention, through the C ABI:
two calls in a row, the second on a smaller cache, each equal to the existing entry point's output
(same kernels, same arithmetic: bit for bit, which is inside the 2e-3 bar) and within 2e-3 of the
oracle; a cache beyond the array's size is refused."""
import numpy as np
import pytest
import torch

from paper_2405_06219_amd import synth

pytestmark = pytest.mark.gpu
D = 128


def test_static_scratch_decode_equals_the_workspace_decode():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import parity_util as P
    B = P.B
    dev = "cuda:0"
    # first a GQA cache cut into many chunks, then a smaller one (fewer heads, fewer tokens, fewer chunks)
    big = synth.Workload("static_big", 2, 16, 4, 9000, 1.5, seed=91)
    little = synth.Workload("static_little", 1, 4, 4, 700, 2.0, seed=92)
    for w in (big, little):
        print("case", w, flush=True)
        pair, k, v, q = P.make_pair(w, extra_tokens=4)
        pair.prefill(k, v)
        pair.append(*synth.make_new_token(w, 0))
        ref = pair.ref.decode(q)
        qd = torch.from_numpy(q).to(dev)
        want = pair.gpu.skvq_decode_attention(qd)
        want16 = torch.empty(q.shape, dtype=torch.float16, device=dev)
        got = torch.full(q.shape, float("nan"), dtype=torch.float32, device=dev)
        got16 = torch.empty(q.shape, dtype=torch.float16, device=dev)
        pair.gpu.skvq_decode_attention(qd, out_f16=want16)
        # poison the caller's workspace: the static variant must not depend on it
        pair.gpu.buffers["workspace"].fill_(0xFF)
        pair.gpu.skvq_decode_attention_static(qd, got, out_f16=got16)
        torch.cuda.synchronize()
        assert bool((pair.gpu.buffers["workspace"] == 0xFF).all())      # ... nor write to it
        got_h, want_h = got.cpu().numpy(), want.cpu().numpy()
        assert np.abs(got_h - want_h).max() <= P.TOL and np.abs(got_h - ref).max() <= P.TOL
        assert np.array_equal(got_h.view(np.uint32), want_h.view(np.uint32))
        assert np.array_equal(got16.cpu().numpy().view(np.uint16), want16.cpu().numpy().view(np.uint16))
    # more (sequence, query head) rows than the array holds: refused, nothing launched
    wide = synth.Workload("static_wide", 3, 32, 32, 200, 1.5, seed=93)
    pair, k, v, q = P.make_pair(wide)
    pair.prefill(k, v)
    out = torch.zeros(q.shape, dtype=torch.float32, device=dev)
    with pytest.raises(B.SkvqError) as e:
        pair.gpu.skvq_decode_attention_static(torch.from_numpy(q).to(dev), out)
    assert e.value.status == B.SKVQ_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
