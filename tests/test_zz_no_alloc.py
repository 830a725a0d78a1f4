"""The entry point that allocates nothing (parle_k_spread_static) against parle_k_spread, through the C ABI.

Both run the same kernels; the only difference is where the per-workgroup partial sums live (the library's
own 32 KiB device array instead of a caller buffer), so the two fp32 results must be bit-identical.  Two
calls in a row, the second on a smaller input: the array keeps the first call's partial sums and the second
call must not read them.  The oracle's spread (float64) bounds both."""
import ctypes as C

import numpy as np
import pytest

from oracle import parle as oparle
from paper_1707_00424_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1707_00424_amd import binding as pb
    pb.lib()
    return torch, pb


def _oracle_spread(x, ref):
    st = oparle.init_state(x, oparle.ParleConfig(n_replicas=x.shape[0]))
    st.x_ref = ref.astype(np.float64)
    return oparle.spread(st)


def test_static_spread_matches_the_scratch_argument_variant(gpu):
    torch, pb = gpu
    # 4 200 004 columns fill all 4096 partial slots; the second input uses 245 of them, the third a single one
    for n, N in [(8, 4_200_004), (3, 250_000), (1, 4)]:
        x = synth.flat_params(21, n, N)
        ref = synth.flat_params(22, 1, N)[0]
        dx, dr = torch.as_tensor(x).cuda(), torch.as_tensor(ref).cuda()
        partial = torch.zeros(4096, dtype=torch.float64, device="cuda")
        want = torch.zeros(1, dtype=torch.float32, device="cuda")
        got = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        print(f"static spread n={n} N={N}", flush=True)
        pb.parle_k_spread(dx, dr, partial, want)
        pb.parle_k_spread_static(dx, dr, got)
        torch.cuda.synchronize()
        assert got.item() == want.item(), (n, N, got.item(), want.item())
        orc = _oracle_spread(x, ref)
        assert abs(got.item() - orc) <= 2e-6 * orc


def test_static_spread_rejects_bad_arguments(gpu):
    torch, pb = gpu
    x = torch.zeros((2, 8), dtype=torch.float32, device="cuda")
    r = torch.zeros(8, dtype=torch.float32, device="cuda")
    out = torch.zeros(1, dtype=torch.float32, device="cuda")
    L = pb.lib()
    too_many = (1 << 34) // 2 + 4                        # 2 * n_pad just above the stated maximum
    assert L.parle_k_spread_static(None, 2, too_many, x.data_ptr(), r.data_ptr(), out.data_ptr()) == pb.PARLE_ESIZE
    assert b"PARLE_SPREAD_STATIC_MAX_ELEMS" in L.parle_last_error(None)
    assert L.parle_k_spread_static(None, 2, 6, x.data_ptr(), r.data_ptr(), out.data_ptr()) == pb.PARLE_EINVAL
    assert L.parle_k_spread_static(None, 2, 8, x.data_ptr(), None, out.data_ptr()) == pb.PARLE_EINVAL
    assert L.parle_k_spread_static(None, 2, 8, x.data_ptr() + 4, r.data_ptr(), out.data_ptr()) == pb.PARLE_EALIGN
    torch.cuda.synchronize()
