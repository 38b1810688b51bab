"""The entry point that allocates nothing (tfno_spectral_conv2d_noalloc) against tfno_spectral_conv2d, through the
C ABI: two calls in a row, the second on a smaller input, both sharing the library's static scratch array."""
import sys

import numpy as np
import pytest

from paper_2504_11681_amd import inputs

pytestmark = pytest.mark.gpu

REL_L2, MAX_ABS = 1e-5, 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_noalloc_entry_point_matches_the_workspace_one_on_two_calls_in_a_row(oracle_mod):
    import torch
    from paper_2504_11681_amd import binding
    assert torch.cuda.is_available(), "this test needs the MI355X"
    L = binding.lib()
    stream = torch.cuda.current_stream().cuda_stream
    # (B, C_in, C_out, N, K): image kernels with a rounded mode count, then a smaller call, then the strip pipeline
    for (B, Ci, Co, N, K) in [(6, 24, 40, 128, 32), (2, 5, 7, 64, 12), (1, 3, 4, 512, 32)]:
        say(f"[case] tfno_spectral_conv2d_noalloc {(B, Ci, Co, N, K)}")
        x = inputs.make_x(2600 + N, B, Ci, (N, N))
        W = inputs.make_W(2600 + N, Ci, Co)
        xd, Wd = torch.from_numpy(x).cuda(), torch.from_numpy(W).cuda()
        need = binding.workspace_bytes(2, 0, B, Ci, Co, N, K)
        assert 0 < need <= binding.NOALLOC_SCRATCH_BYTES
        y_new = torch.full((B, Co, N, N), float("nan"), dtype=torch.complex64, device="cuda")
        st = L.tfno_spectral_conv2d_noalloc(xd.data_ptr(), Wd.data_ptr(), y_new.data_ptr(), B, Ci, Co, N, K, stream)
        assert st == binding.OK, binding.status_string(st)
        torch.cuda.synchronize()
        y_old = torch.full((B, Co, N, N), float("nan"), dtype=torch.complex64, device="cuda")
        binding.spectral_conv2d(xd, Wd, y_old, K)              # the existing entry point, registered workspace
        torch.cuda.synchronize()
        got, ref = y_new.cpu().numpy().astype(np.complex128), y_old.cpu().numpy().astype(np.complex128)
        assert not np.isnan(got.view(np.float64)).any(), "some outputs were never written"
        rel = np.linalg.norm((got - ref).ravel()) / np.linalg.norm(ref.ravel())
        mx = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
        say(f"   against tfno_spectral_conv2d: rel_l2={rel:.3e} max_abs/max|y|={mx:.3e} "
            f"bitwise_equal={np.array_equal(y_new.cpu().numpy().view(np.float32), y_old.cpu().numpy().view(np.float32))}")
        assert rel <= REL_L2 and mx <= MAX_ABS
        want, _ = oracle_mod.spectral_conv2d(x, W, K)
        rel = np.linalg.norm((got - want).ravel()) / np.linalg.norm(want.ravel())
        mx = np.max(np.abs(got - want)) / np.max(np.abs(want))
        say(f"   against the oracle: rel_l2={rel:.3e} max_abs/max|y|={mx:.3e}")
        assert rel <= REL_L2 and mx <= MAX_ABS
    # a shape beyond the scratch array is refused before any launch
    B, Ci, Co, N, K = 32, 64, 64, 256, 64
    assert binding.workspace_bytes(2, 0, B, Ci, Co, N, K) > binding.NOALLOC_SCRATCH_BYTES
    big = torch.empty(1, dtype=torch.complex64, device="cuda")
    st = L.tfno_spectral_conv2d_noalloc(0x10000000, 0x10000000 + (1 << 40), 0x10000000 + (2 << 40), B, Ci, Co, N, K, stream)
    assert st == binding.ERR_WORKSPACE
    del big
    torch.cuda.synchronize()
