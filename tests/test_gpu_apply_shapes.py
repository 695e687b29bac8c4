"""The two launch shapes of the apply pass give the same bits: a vector long
enough for the LDS-staged kernel (one block per compute unit, slabs of results)
against the direct kernel run on slices of the same rows, for every compiled-in
worker count, a run-time one, the three storage types, ragged lengths and both
modes (eq. (2) step and the operator of eq. (4) on a vector z)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1709_05069_amd as qn
from parity_util import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SLAB_ROWS = 32768


def _staged_rows():
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    return SLAB_ROWS * cus          # from here on the staged kernel runs


CASES = [(4, torch.float32, 3), (8, torch.float32, 1), (16, torch.float32, 2), (32, torch.float32, 5),
         (64, torch.float32, 0), (24, torch.float32, 7), (1, torch.float32, 1), (33, torch.float32, 6),
         (32, torch.bfloat16, 9), (16, torch.bfloat16, 0), (5, torch.bfloat16, 11), (32, torch.float16, 4)]


@pytest.mark.parametrize("m,storage,extra", CASES)
def test_staged_and_direct_kernels_agree_bit_for_bit(m, storage, extra):
    n = _staged_rows() + 70_000 + extra            # a partial last slab and a ragged tail
    g = torch.Generator(device=DEV).manual_seed(100 * m + extra)
    base = torch.randn(n, device=DEV, generator=g)
    th = torch.empty((m, n), dtype=storage, device=DEV)
    gr = torch.empty((m, n), dtype=storage, device=DEV)
    for k in range(m):                              # row by row: no (m, n) fp32 temporaries
        th[k] = (base + 1e-2 * torch.randn(n, device=DEV, generator=g)).to(storage)
        gr[k] = (2.0 * base - 1.0 + 1e-2 * torch.randn(n, device=DEV, generator=g)).to(storage)
    c = torch.linspace(-0.7, 1.1, m, device=DEV)
    z = torch.randn(n, device=DEV, generator=g)
    full = qn.qn_apply(th, gr, c, 0.6)
    full_z = qn.qn_hinv_apply(th, gr, z, c)
    torch.cuda.synchronize()
    # slices far below the staged threshold take the direct kernel: slab and round
    # boundaries of the staged launch, the ragged end, the start
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    starts = [0, SLAB_ROWS - 8, SLAB_ROWS * (cus - 1) - 4, SLAB_ROWS * cus - 12, n - 40_000]
    for r0 in starts:
        r0 -= r0 % 8                                # keep the slices' columns 16-byte aligned
        rows = min(40_000, n - r0)
        part = qn.qn_apply(th[:, r0:r0 + rows], gr[:, r0:r0 + rows], c, 0.6)
        assert torch.equal(part, full[r0:r0 + rows]), (m, storage, r0)
        pz = qn.qn_hinv_apply(th[:, r0:r0 + rows], gr[:, r0:r0 + rows],
                              z[r0:r0 + rows].contiguous(), c)
        assert torch.equal(pz, full_z[r0:r0 + rows]), (m, storage, r0, "z")
    # and the last rows against the oracle
    r0 = n - 5000
    ref = oracle.apply_closed_form(th[:, r0:].float().cpu().numpy().astype(np.float64),
                                   gr[:, r0:].float().cpu().numpy().astype(np.float64),
                                   c.double().cpu().numpy(), 0.6)
    assert_close(full[r0:].cpu().numpy(), ref, 2e-6 if storage == torch.float32 else 1e-3, k=4.0)
