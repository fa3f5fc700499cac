"""The entry point that allocates nothing (pm_conv3x3_bwd_weight_static: partial results in the library's
fixed device array) against the entry point it is a variant of (pm_conv3x3_bwd_weight with a caller
workspace), through the C ABI: two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared array must not leak into the second result.  Same kernels, same
partial-sum order: the results must be bit-identical."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _case(torch, pm, dtype, B, H, Cin, Cout, stride, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Ho = (H - 1) // stride + 1
    x = torch.randn((B, H, H, Cin), generator=g).to(tdt).cuda()
    dz = torch.randn((B, Ho, Ho, Cout), generator=g).to(tdt).cuda()
    n = Cout * 9 * Cin
    ref = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    nscr = pm.pm_conv3x3_bwd_weight_scratch(dtype, B, H, H, Cin, Cout, stride)
    scr = torch.empty(max(nscr, 4), dtype=torch.uint8, device="cuda")
    pm.pm_conv3x3_bwd_weight(st, dtype, B, H, H, Cin, Cout, stride, dz.data_ptr(), x.data_ptr(), ref.data_ptr(),
                             scr.data_ptr(), nscr)
    pm.pm_conv3x3_bwd_weight_static(st, dtype, B, H, H, Cin, Cout, stride, dz.data_ptr(), x.data_ptr(), got.data_ptr())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(ref).all())
    assert torch.equal(ref, got), float((ref - got).abs().max())
    return nscr, ref.cpu().numpy().astype(np.float64), x, dz


def test_static_scratch_entry_point_matches_workspace_entry_point():
    import torch
    import paper_1910_05124_amd as pm
    assert torch.cuda.is_available()
    cap = pm.pm_static_scratch_bytes()
    assert cap == 16 << 20
    # first call: large maps (MFMA path, four chunks per wave, 2.4 MB of partial results)
    n1, dW1, x1, dz1 = _case(torch, pm, "bf16", 128, 32, 16, 16, 1, seed=1)
    assert 0 < n1 <= cap
    # second call right after it, smaller input and another kernel variant (one tap row per block)
    n2, dW2, _, _ = _case(torch, pm, "bf16", 8, 8, 32, 64, 1, seed=2)
    assert 0 < n2 < n1
    # the image layer (thin kernels) and a stride-2 layer
    _case(torch, pm, "bf16", 16, 32, 3, 16, 1, seed=3)
    _case(torch, pm, "bf16", 16, 16, 16, 32, 2, seed=4)
    # a shape on the plain path needs no partial results at all
    n5, _, _, _ = _case(torch, pm, "f32", 2, 6, 8, 8, 1, seed=5)
    assert n5 == 0
    # the first result against the definition (correlation of dz with x), so both entry points are right
    X = x1.float().cpu().numpy().astype(np.float64)
    DZ = dz1.float().cpu().numpy().astype(np.float64)
    Xp = np.pad(X, ((0, 0), (1, 1), (1, 1), (0, 0)))
    want = np.zeros((16, 9, 16))
    for t in range(9):
        dy, dx = divmod(t, 3)
        want[:, t, :] = np.einsum("bhwo,bhwi->oi", DZ, Xp[:, dy:dy + 32, dx:dx + 32, :])
    assert np.max(np.abs(dW1 - want.ravel())) / np.max(np.abs(want)) <= 3e-6


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    import paper_1910_05124_amd as pm
    B, H, Cin, Cout = 128, 32, 64, 64            # 256 blocks x 36864 partial values x 4 B = 37.7 MB > 16 MiB
    need = pm.pm_conv3x3_bwd_weight_scratch("bf16", B, H, H, Cin, Cout, 1)
    assert need > pm.pm_static_scratch_bytes()
    x = torch.zeros((B, H, H, Cin), dtype=torch.bfloat16, device="cuda")
    dz = torch.zeros((B, H, H, Cout), dtype=torch.bfloat16, device="cuda")
    dW = torch.full((Cout * 9 * Cin,), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(pm.PmError) as e:
        pm.pm_conv3x3_bwd_weight_static(torch.cuda.current_stream().cuda_stream, "bf16", B, H, H, Cin, Cout, 1,
                                        dz.data_ptr(), x.data_ptr(), dW.data_ptr())
    assert e.value.name == "PM_ENOMEM"
    torch.cuda.synchronize()
    assert bool((dW == 7.0).all())               # nothing was launched
    with pytest.raises(pm.PmError):
        pm.pm_conv3x3_bwd_weight_static(None, "bf16", B, H, H, Cin, Cout, 3, dz.data_ptr(), x.data_ptr(), dW.data_ptr())
