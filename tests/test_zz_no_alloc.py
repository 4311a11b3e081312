"""`sig_forward_chunked_static` (the entry point that allocates nothing: its scratch memory is a fixed array inside the
library) against `sig_forward_chunked` with a caller's workspace, through the C ABI on raw device pointers: two
calls in a row on the same GPU, the second with a smaller input, so that the second finds the first one's leftovers
in the shared array."""
import numpy as np
import pytest

import paper_2001_00706_amd as sig
from oracle import sig_oracle as orc
from paper_2001_00706_amd.inputs import brownian_paths

pytestmark = pytest.mark.gpu


def both_ways(x, N, chunks):
    """(static scratch, caller's workspace) results of the same chunked scan, C calls on raw pointers."""
    import torch
    lib = sig.load_library()
    B, L, d = x.shape
    S = sig.sig_signature_channels(d, N)
    xt = torch.from_numpy(x).to("cuda:0")
    hs = torch.cuda.current_stream().cuda_stream
    need = sig.sig_forward_chunked_workspace_bytes(B, L, d, N, False, chunks, sig.SIG_F32)
    assert 0 < need <= sig.sig_forward_chunked_static_max_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    want = torch.full((B, S), float("nan"), device="cuda:0")
    got = torch.full((B, S), float("nan"), device="cuda:0")
    st = lib.sig_forward_chunked(xt.data_ptr(), B, L, d, N, 0, 0, chunks, sig.SIG_F32, want.data_ptr(), ws.data_ptr(), need, hs)
    assert st == sig.SIG_OK
    st = lib.sig_forward_chunked_static(xt.data_ptr(), B, L, d, N, 0, 0, chunks, sig.SIG_F32, got.data_ptr(), hs)
    assert st == sig.SIG_OK
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


def test_two_calls_in_a_row_the_second_smaller():
    for B, L, d, N, chunks in [(6, 300, 4, 6, 16), (2, 70, 4, 6, 4)]:
        x = brownian_paths(B, L, d, seed=B + L)
        got, want = both_ways(x, N, chunks)
        assert np.all(np.isfinite(got))
        np.testing.assert_array_equal(got, want)          # same kernels, same order of operations: same bits
        ref = orc.signature(x, N)
        for sl in orc.level_slices(d, N):
            assert np.linalg.norm(got[:, sl] - ref[:, sl]) <= 1e-4 * np.linalg.norm(ref[:, sl])


def test_other_kernel_families_and_fp64():
    import torch
    for B, L, d, N, chunks, dtype in [(3, 50, 2, 6, 8, np.float32), (2, 40, 5, 3, 4, np.float64), (2, 90, 8, 4, 2, np.float32)]:
        x = brownian_paths(B, L, d, seed=L).astype(dtype)
        xt = torch.from_numpy(x).to("cuda:0")
        got = sig.sig_forward_chunked_static(xt, N, chunks)
        want = sig.sig_forward_chunked(xt, N, chunks)
        torch.cuda.synchronize()
        assert torch.equal(got, want)


def test_requests_beyond_the_fixed_scratch_are_refused_and_leave_the_output_alone():
    import torch
    limit = sig.sig_forward_chunked_static_max_bytes()
    assert limit == 32 * 1024 * 1024
    B, L, d, N, chunks = 8, 4000, 4, 6, 256        # 1.5 * 8 * 256 signatures of 5460 floats = 67 MB
    assert sig.sig_forward_chunked_workspace_bytes(B, L, d, N, False, chunks, sig.SIG_F32) > limit
    x = torch.zeros((B, L, d), device="cuda:0")
    out = torch.full((B, sig.sig_signature_channels(d, N)), 7.0, device="cuda:0")
    with pytest.raises(sig.SigError) as e:
        sig.sig_forward_chunked_static(x, N, chunks, out=out)
    assert e.value.status == sig.SIG_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert bool(torch.all(out == 7.0))
    with pytest.raises(sig.SigError) as e:
        sig.sig_forward_chunked_static(x, N, 3, out=out)      # not a power of two
    assert e.value.status == sig.SIG_ERR_INVALID_ARG
