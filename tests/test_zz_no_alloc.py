"""lfmmi_loss_grad_static (the entry point for callers that cannot allocate: its workspace is scratch memory built
into the library) against lfmmi_loss_grad with a caller's workspace, through the C-ABI: two calls in a row on the
shared scratch memory, the second on a smaller input; sizes beyond the built-in memory are refused."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2112_00709_amd as lib
    lib.lib()
    return lib


def run_both(fb, w):
    import torch
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    emis = torch.from_numpy(w.emis).cuda()
    lengths = torch.from_numpy(w.lengths.astype(np.int32)).cuda()
    need = fb.fb_lfmmi_workspace_bytes(Gd, Gn, w.B, w.N, w.D)
    assert 0 < need <= fb.fb_static_scratch_bytes()
    ws = torch.full((need,), 255, dtype=torch.uint8, device="cuda")
    grad = torch.full((w.B, w.N, w.D), float("nan"), dtype=torch.float32, device="cuda")
    want = [x.cpu().numpy().copy() for x in fb.lfmmi_loss_grad(Gd, Gn, emis, lengths, ws=ws, grad=grad)]
    outs = (torch.full((1,), float("nan"), dtype=torch.float64, device="cuda"),
            torch.full((w.B,), float("nan"), dtype=torch.float64, device="cuda"),
            torch.full((w.B,), float("nan"), dtype=torch.float64, device="cuda"),
            torch.full((w.B, w.N, w.D), float("nan"), dtype=torch.float32, device="cuda"))
    fb.lfmmi_loss_grad_static(Gd, Gn, emis, lengths, *outs)
    torch.cuda.synchronize()
    got = [x.cpu().numpy() for x in outs]
    Gd.destroy(); Gn.destroy()
    return want, got


def test_static_scratch_matches_workspace_call(fb):
    # a denominator large enough for the 16-wave kernels, a ragged batch in length groups; then a smaller problem of
    # another shape on the same scratch memory (small graph kernels, one launch per stage)
    for w in (wl.config5(K=1500, B=36, Lmin=2, Lmax=8, D=120), wl.config5(K=300, B=6, Lmin=2, Lmax=9, D=40)):
        want, got = run_both(fb, w)
        for i, (a, b) in enumerate(zip(want, got)):
            assert np.isfinite(b).all()
            if i < 3:
                assert np.array_equal(a, b)          # objective and log Z: the same kernels on the same inputs
            else:
                np.testing.assert_allclose(b, a, rtol=0, atol=3e-6)   # gradient: sums of the same terms
        # the objective against its definition from the two log Z vectors
        assert abs(got[0][0] - (got[1] - got[2])[w.lengths > 0].sum()) <= 1e-9 * max(1.0, abs(got[0][0]))


def test_static_scratch_refuses_what_does_not_fit(fb):
    import torch
    w = wl.config5(K=1500, B=64, Lmin=30, Lmax=60, D=200)
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    assert fb.fb_lfmmi_workspace_bytes(Gd, Gn, w.B, w.N, w.D) > fb.fb_static_scratch_bytes()
    emis = torch.from_numpy(w.emis).cuda()
    lengths = torch.from_numpy(w.lengths.astype(np.int32)).cuda()
    outs = (torch.zeros((1,), dtype=torch.float64, device="cuda"), torch.zeros((w.B,), dtype=torch.float64, device="cuda"),
            torch.zeros((w.B,), dtype=torch.float64, device="cuda"), torch.zeros((w.B, w.N, w.D), dtype=torch.float32, device="cuda"))
    with pytest.raises(fb.FBError) as err:
        fb.lfmmi_loss_grad_static(Gd, Gn, emis, lengths, *outs)
    assert err.value.code == fb.FB_EUNSUPPORTED and "workspace" in str(err.value)
    Gd.destroy(); Gn.destroy()
