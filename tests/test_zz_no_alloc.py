"""dr_csr_normalize_noalloc (the entry point for callers that cannot allocate: its scratch is a device array inside the
library image) against dr_csr_normalize, bit for bit, through the C ABI: two calls in a row on one GPU, the second on a
smaller input, so that what the first call left in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

import paper_2508_16769_amd as P
from gpu_util import dev, random_csr, say

pytestmark = pytest.mark.gpu


def _both(mode, M, N, rowptr, colidx):
    rp, ci = dev(rowptr), dev(colidx)
    want = torch.full((len(colidx),), -1.0, dtype=torch.float32, device="cuda")
    got = torch.full((len(colidx),), -2.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(256, P.dr_csr_normalize_workspace_bytes(mode, M, N, len(colidx))), dtype=torch.uint8, device="cuda")
    P.dr_csr_normalize(mode, M, N, rp, ci, want, ws)
    P.dr_csr_normalize_noalloc(mode, M, N, rp, ci, got)
    torch.cuda.synchronize()
    return got.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32)


def test_noalloc_matches_workspace_variant_on_two_calls_in_a_row():
    rng = np.random.default_rng(77)
    # first call: many columns with high counts; second call: fewer rows and columns, sparser
    for label, (M, N, max_deg) in (("first, larger", (5000, 3000, 40)), ("second, smaller", (700, 450, 6))):
        rowptr, colidx, _ = random_csr(rng, M, N, max_deg, dup=True)
        say(f"dr_csr_normalize_noalloc {label}: M={M} N={N} nnz={len(colidx)}")
        for mode in (P.DR_NORM_SYM, P.DR_NORM_MEAN):
            got, want = _both(mode, M, N, rowptr, colidx)
            assert np.array_equal(got, want), (label, mode)


def test_noalloc_rejects_sizes_beyond_its_scratch():
    import ctypes
    lib = P.load()
    one = ctypes.c_void_p(256)
    big = (1 << 21) + 1
    rc = lib.dr_csr_normalize_noalloc(P.DR_NORM_SYM, ctypes.c_int64(4), ctypes.c_int64(big), ctypes.c_int64(5), one, one, one, None)
    assert rc == P.DR_ERR_UNSUPPORTED and "DR_NOALLOC_MAX_COLS" in P.dr_last_error()
