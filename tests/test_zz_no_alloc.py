"""ec_row_entropy_noalloc (the entry point that allocates nothing: its partial tuples live in
an array of the library's device image) against ec_row_entropy, through the C ABI: same kernels,
so the results must be bit-identical; two calls in a row, the second with a smaller input, so
that what the first left in the shared array cannot leak into the second."""
import numpy as np
import pytest
import torch

import paper_2603_18489_amd as ec

pytestmark = pytest.mark.gpu


def test_noalloc_matches_workspace_variant_on_two_calls_in_a_row():
    rng = np.random.default_rng(5)
    big = torch.from_numpy((rng.standard_normal((128, 126464)) * 6.0).astype(np.float32)).cuda()
    small = torch.from_numpy((rng.standard_normal((5, 4100)) * 9.0).astype(np.float32)).cuda()
    out_big = torch.full((128, 4), -1.0, dtype=torch.float32, device="cuda")
    out_small = torch.full((5, 4), -1.0, dtype=torch.float32, device="cuda")
    # reference results from the variant whose scratch is a caller-provided workspace
    ref_big = ec.row_entropy(big).cpu().numpy()
    ref_small = ec.row_entropy(small).cpu().numpy()
    # the first call on a device looks up the array's address (set-up); after it, no call may
    # change the amount of free device memory
    ec.row_entropy_noalloc(small, out_small)
    torch.cuda.synchronize()
    out_small.fill_(-1.0)
    free0 = torch.cuda.mem_get_info()[0]
    ec.row_entropy_noalloc(big, out_big)
    ec.row_entropy_noalloc(small, out_small)      # same stream: ordered after the first call
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0, "the call must not allocate device memory"
    assert np.array_equal(out_big.cpu().numpy(), ref_big)
    assert np.array_equal(out_small.cpu().numpy(), ref_small)
    assert (ref_big[:, 2] > 0).all() and (ref_small[:, 1] > 0).all()
    # and once more in the other order
    out_big.fill_(-1.0)
    ec.row_entropy_noalloc(small, out_small)
    ec.row_entropy_noalloc(big, out_big)
    torch.cuda.synchronize()
    assert np.array_equal(out_big.cpu().numpy(), ref_big)
    assert np.array_equal(out_small.cpu().numpy(), ref_small)


def test_noalloc_rejects_sizes_beyond_its_scratch():
    z = torch.zeros((2, 4096), dtype=torch.float32, device="cuda")
    lib = ec.load_library()
    import ctypes as C
    out = torch.zeros((2, 4), dtype=torch.float32, device="cuda")
    vp = C.c_void_p
    assert lib.ec_row_entropy_noalloc(vp(z.data_ptr()), ec.EC_MAX_BLOCK + 1, 4096, 4096,
                                      vp(out.data_ptr()), None) == ec.EC_ERR_ARG
    assert lib.ec_row_entropy_noalloc(vp(z.data_ptr()), 2, 163841, 163841, vp(out.data_ptr()),
                                      None) == ec.EC_ERR_ARG
    assert lib.ec_row_entropy_noalloc(None, 2, 4096, 4096, vp(out.data_ptr()), None) == ec.EC_ERR_ARG
