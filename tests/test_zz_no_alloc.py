"""The stored-noise entry point that allocates no device memory (its table lives in a fixed
device array of the library) against the allocating entry point it is a variant of: identical
draws, on two calls in a row that share the array, the second with a smaller table and output."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def isr():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2108_09413_amd as lib
    return lib


def test_static_table_entry_point_matches_the_allocating_one(isr):
    import torch
    print("no-allocation stored-noise entry point", flush=True)
    assert isr.lib().isr_noise_bank_static_capacity() == 64 * 1024
    # first call: the largest table that fits (sigma 380 -> about 61 KiB), a ragged tensor size;
    # second call: a much smaller table (sigma 8) and output, reading the array the first one filled;
    # third: back to a mid-sized one
    for sigma, seed, bank, first, count, d in ((380, 7, 3, 4090, 9, 3 * 32 * 32), (8, 7, 3, 0, 2, 12),
                                              (128, 0xFFFFFFFF00000001, 0, 5, 4, 3 * 32 * 32)):
        want = isr.isr_noise_bank(sigma, seed, bank, first, count, d)
        out = torch.full((count, d), -12345, dtype=torch.int16, device="cuda")
        got = isr.isr_noise_bank_static(sigma, seed, bank, first, count, d, out)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (sigma, count, d)
        # draws of the discrete Gaussian on the lattice: not the fill value, spread about sigma
        g = got.to(torch.float64)
        assert abs(float(g.std()) / sigma - 1.0) < (0.5 if count * d < 100 else 0.05)
    # a sigma whose table exceeds the fixed array is refused, without touching the output
    out = torch.full((1, 8), 77, dtype=torch.int16, device="cuda")
    rc = isr.lib().isr_noise_bank_static(1024, ctypes.c_uint64(0), 0, 0, 1, 8, ctypes.c_void_p(out.data_ptr()), None)
    assert rc == isr.ISR_ERR_WORKSPACE and bool((out == 77).all())
    for bad_sigma, bad_d in ((0, 8), (1025, 8), (32, 6), (32, 0)):
        rc = isr.lib().isr_noise_bank_static(bad_sigma, ctypes.c_uint64(0), 0, 0, 1, bad_d, ctypes.c_void_p(out.data_ptr()), None)
        assert rc == isr.ISR_ERR_ARG
    assert isr.lib().isr_noise_bank_static(32, ctypes.c_uint64(0), 0, 0, 1, 8, None, None) == isr.ISR_ERR_ARG
    # and the array is still good afterwards
    want = isr.isr_noise_bank(32, 1, 2, 3, 4, 16)
    got = isr.isr_noise_bank_static(32, 1, 2, 3, 4, 16, torch.empty((4, 16), dtype=torch.int16, device="cuda"))
    assert torch.equal(got, want)
