"""The comparison entry point that allocates nothing (opevo_compare_f32_static): its partial
results live in device memory that is part of the library's code object.  Checked against
opevo_compare_f32 (same kernel, host-side fold) on two calls in a row, the second on a smaller
input, through the C ABI."""
import numpy as np
import pytest

import paper_2006_05664_amd as P

pytestmark = pytest.mark.gpu


def test_static_compare_matches_the_allocating_one_twice_in_a_row():
    import torch
    assert torch.cuda.is_available()
    stream = torch.cuda.current_stream().cuda_stream
    result = torch.full((2,), float("nan"), dtype=torch.float64, device="cuda:0")
    g = torch.Generator(device="cpu").manual_seed(20240611)
    # the first input spans all 1024 workgroups with a ragged tail, the second only 4 of them: what
    # the first call left in the other partials must not reach the second result
    for n, scale in (((1 << 22) + 12345, 1e-3), (1000, 5e-2)):
        ref = torch.randn(n, generator=g, dtype=torch.float32)
        c = ref + scale * torch.randn(n, generator=g, dtype=torch.float32)
        dref, dc = ref.cuda(), c.cuda()
        want = P.opevo_compare_f32(dc.data_ptr(), dref.data_ptr(), n, stream)
        P.opevo_compare_f32_static(dc.data_ptr(), dref.data_ptr(), n, stream, result.data_ptr())
        torch.cuda.synchronize()
        got = result.cpu().numpy()
        # same partials, same fold order: max is exact; the ratio and root are IEEE operations on both sides
        assert got[0] == want[0], (n, got, want)
        assert abs(got[1] - want[1]) <= 1e-12 * want[1], (n, got, want)
        # and both agree with the definition evaluated in fp64 on the host
        r64, c64 = ref.double().numpy(), c.double().numpy()
        mx = np.max(np.abs(c64 - r64) / (np.abs(r64) + 1.0))
        fro = np.linalg.norm(c64 - r64) / np.linalg.norm(r64)
        assert abs(got[0] - mx) <= 1e-12 * mx and abs(got[1] - fro) <= 1e-9 * fro, (n, got, mx, fro)
    # a NaN in c can never pass
    dc[n // 2] = float("nan")
    P.opevo_compare_f32_static(dc.data_ptr(), dref.data_ptr(), n, stream, result.data_ptr())
    torch.cuda.synchronize()
    assert np.isinf(result.cpu().numpy()[0])


def test_static_compare_refuses_sizes_beyond_its_limit():
    import torch
    assert torch.cuda.is_available()
    buf = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    result = torch.zeros(2, dtype=torch.float64, device="cuda:0")
    with pytest.raises(P.OpevoError) as e:
        P.opevo_compare_f32_static(buf.data_ptr(), buf.data_ptr(), (1 << 34) + 1, 0, result.data_ptr())
    assert e.value.status == P.OPEVO_E_ARG and "limit" in e.value.message
    with pytest.raises(P.OpevoError):
        P.opevo_compare_f32_static(buf.data_ptr(), buf.data_ptr(), 16, 0, 0)
