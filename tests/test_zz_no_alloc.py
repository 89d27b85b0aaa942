"""The PLP step for callers that cannot allocate: plp_step_static runs plp_step's kernels on the
library's own static scratch array.  Called through the C ABI, its results have to be the bits of
plp_step on a caller's workspace -- on two calls in a row, the second with a smaller batch (the array
keeps the first call's contents) -- and sizes beyond the array are refused before any launch."""
import math

import numpy as np
import pytest

from paper_2602_11812_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2602_11812_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load_library()
    return binding


def _bits(t):
    return t.cpu().numpy().view(np.int32)


def test_static_step_reproduces_plp_step_on_two_calls_in_a_row(gpu):
    import torch
    spec = wl.scaled(wl.SPECS["plp_decode"], seed=171, B=300, d=512, V=5000, d_h=96, lengths=tuple([1] * 300))
    w = wl.make(spec)
    td = gpu.to_device
    sc = gpu.Scorer(td(w.w_lm), gpu.make_head(td(w.w1), td(w.w2)))
    d = spec.d
    assert gpu.egtp_static_scratch_bytes() == 64 << 20

    def fresh(S):
        return (torch.zeros(S, d, dtype=torch.float32, device="cuda"),
                torch.full((S,), -math.inf, dtype=torch.float32, device="cuda"))

    # call 1: one token for each of 300 sequences; call 2: a ragged chunk for 7 of them through `slot`
    g1 = td(wl.decode_hidden(spec, 1))
    chunk_len = np.array([3, 0, 64, 1, 17, 5, 2], dtype=np.int32)
    coff = np.concatenate([[0], np.cumsum(chunk_len)]).astype(np.int32)
    g2 = td(wl.decode_hidden(spec, 2, rows=int(coff[-1])))
    slot = torch.tensor([250, 3, 17, 299, 0, 42, 8], dtype=torch.int32).cuda()
    coff_dev = torch.from_numpy(coff).cuda()

    results = {}
    for which in ("workspace", "static"):
        pooled, lse = fresh(300)
        e1 = torch.empty(300, dtype=torch.float32, device="cuda")
        r1 = torch.empty(300, dtype=torch.float32, device="cuda")
        e2 = torch.empty(int(coff[-1]), dtype=torch.float32, device="cuda")
        r2 = torch.empty(7, dtype=torch.float32, device="cuda")
        if which == "workspace":
            gpu.plp_step(sc.ctx, g1, None, None, None, 300, 300, pooled, lse, sc.workspace(300, 300), e1, r1)
            gpu.plp_step(sc.ctx, g2, coff_dev, coff, slot, 7, int(coff[-1]), pooled, lse,
                         sc.workspace(int(coff[-1]), 7), e2, r2)
        else:
            gpu.plp_step_static(sc.ctx, g1, None, None, None, 300, 300, pooled, lse, e1, r1)
            gpu.plp_step_static(sc.ctx, g2, coff_dev, coff, slot, 7, int(coff[-1]), pooled, lse, e2, r2)
        torch.cuda.synchronize()
        results[which] = [_bits(t) for t in (e1, r1, e2, r2, pooled, lse)]
    for name, a, b in zip(("entropy 1", "prediction 1", "entropy 2", "prediction 2", "pooled", "lse"),
                          results["workspace"], results["static"]):
        assert np.array_equal(a, b), name
    assert np.isfinite(results["static"][1].view(np.float32)).all()
    sc.close()


def test_static_step_refuses_what_does_not_fit(gpu):
    import torch
    spec = wl.scaled(wl.SPECS["plp_decode"], seed=173, B=4, d=256, V=3000, d_h=32, lengths=(1, 1, 1, 1))
    w = wl.make(spec)
    td = gpu.to_device
    sc = gpu.Scorer(td(w.w_lm), gpu.make_head(td(w.w1), td(w.w2)))
    big_T = 1 << 20                                        # the packed copy of the hidden states alone is 512 MiB
    assert gpu.egtp_workspace_bytes(sc.ctx, big_T, 4) > gpu.egtp_static_scratch_bytes()
    pooled = torch.zeros(4, spec.d, dtype=torch.float32, device="cuda")
    lse = torch.full((4,), -math.inf, dtype=torch.float32, device="cuda")
    pred = torch.full((4,), 7.0, dtype=torch.float32, device="cuda")
    off = torch.tensor([0, 1, 2, 3, big_T], dtype=torch.int32).cuda()
    fake_hidden = td(wl.decode_hidden(spec, 1))            # never read: the call is refused on its sizes
    with pytest.raises(gpu.EgtpError) as e:
        gpu.plp_step_static(sc.ctx, fake_hidden, off, None, None, 4, big_T, pooled, lse, None, pred)
    assert e.value.status == 5
    torch.cuda.synchronize()
    assert bool((pred == 7.0).all()) and not bool(pooled.any())     # nothing was launched
    gpu.plp_step_static(sc.ctx, fake_hidden, None, None, None, 4, 4, pooled, lse, None, pred)   # a fitting call works
    torch.cuda.synchronize()
    assert bool(torch.isfinite(pred).all())
    sc.close()
