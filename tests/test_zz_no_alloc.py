"""fax_cross_entropy_static: the loss and its gradient for callers that cannot allocate.  Its
per-row scratch is an array built into the library; the results must be those of
fax_cross_entropy (which takes that scratch from the caller) bit for bit, on two calls in a row
that share the array, the second with fewer rows than the first left behind, and it must refuse
more rows than the array holds without enqueuing anything."""
import numpy as np
import pytest
import torch

import paper_2204_06514_amd as fax
from oracle import transformer as orc
from helpers import DEV, to_np

pytestmark = pytest.mark.gpu


def _logits(N, V, dtype, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    z = (3.0 * torch.randn(N, V, generator=g)).to(dtype).to(DEV)
    y = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(DEV)
    return z, y


def _both(N, V, dtype, seed):
    z, y = _logits(N, V, dtype, seed)
    code = fax.dtype_code(dtype)
    d_ref = torch.empty_like(z); rows = torch.full((N,), -1.0, device=DEV); loss_ref = torch.zeros(4, device=DEV)
    fax.fax_cross_entropy(code, N, V, z, y, d_ref, rows, loss_ref)
    d_new = torch.empty_like(z); loss_new = torch.zeros(4, device=DEV)
    fax.fax_cross_entropy_static(code, N, V, z, y, d_new, loss_new)
    torch.cuda.synchronize()
    assert torch.equal(d_new, d_ref), (N, V)
    assert loss_new[0].item() == loss_ref[0].item(), (N, V)
    return z, y, d_new, loss_new[0].item()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32], ids=["bf16", "f32"])
def test_two_calls_in_a_row_the_second_smaller(dtype):
    # 1536 rows, then 200 rows: the second call finds 1336 stale per-row losses behind its own
    z1, y1, d1, l1 = _both(1536, 4096, dtype, seed=1)
    z2, y2, d2, l2 = _both(200, 1000, dtype, seed=2)
    # and against the oracle, at the bar of one rounding of the stored gradient
    for z, y, d, l in ((z1, y1, d1, l1), (z2, y2, d2, l2)):
        loss_ref, dz_ref = orc.cross_entropy(to_np(z), y.cpu().numpy().astype(np.int64))
        assert abs(l - loss_ref) <= 1e-5 * abs(loss_ref)
        got = to_np(d)
        bar = 4e-3 if dtype == torch.bfloat16 else 1e-5
        assert np.linalg.norm(got - dz_ref) <= bar * np.linalg.norm(dz_ref)


def test_in_place_and_row_limit():
    z, y = _logits(64, 512, torch.bfloat16, seed=3)
    want = torch.empty_like(z); rows = torch.empty(64, device=DEV); l0 = torch.zeros(4, device=DEV)
    fax.fax_cross_entropy(fax.FAX_BF16, 64, 512, z, y, want, rows, l0)
    l1 = torch.zeros(4, device=DEV)
    fax.fax_cross_entropy_static(fax.FAX_BF16, 64, 512, z, y, z, l1)   # gradient written over the logits
    torch.cuda.synchronize()
    assert torch.equal(z, want) and l0[0].item() == l1[0].item()
    limit = fax.fax_cross_entropy_static_max_rows()
    assert limit == 1 << 18
    before = z.clone()
    with pytest.raises(fax.FaxError) as e:
        fax.fax_cross_entropy_static(fax.FAX_BF16, limit + 1, 512, z, y, z, l1)
    assert e.value.status == fax.FAX_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.equal(z, before)
