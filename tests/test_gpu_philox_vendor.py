"""Known-answer check of the oracle's Philox-4x32-10 against the GPU vendor's random-number library
(an independent implementation of the published generator).  It needs a GPU only because that
library allocates through the HIP runtime; the stream compared is the oracle's, computed on the CPU."""
import ctypes
import os

import numpy as np
import pytest

from oracle import philox

pytestmark = pytest.mark.gpu
_LIB = "/opt/rocm/lib/librocrand.so"
_PHILOX4_32_10 = 404          # generator type code of the library's C API


def test_oracle_words_equal_the_vendor_generator(lib):
    if not os.path.exists(_LIB):
        pytest.skip("vendor random-number library not installed")
    import torch
    rr = ctypes.CDLL(_LIB)
    gen = ctypes.c_void_p()
    assert rr.rocrand_create_generator(ctypes.byref(gen), _PHILOX4_32_10) == 0
    try:
        for seed in (0x1234567890ABCDEF, 7):
            assert rr.rocrand_set_seed(gen, ctypes.c_ulonglong(seed)) == 0
            assert rr.rocrand_set_offset(gen, ctypes.c_ulonglong(0)) == 0
            n = 4096
            out = torch.zeros(n, dtype=torch.int32, device="cuda:0")
            assert rr.rocrand_generate(gen, ctypes.c_void_p(out.data_ptr()), ctypes.c_size_t(n)) == 0
            torch.cuda.synchronize()
            got = out.cpu().numpy().view(np.uint32)
            # the library numbers its blocks by the first counter word, key = the seed's two halves
            blocks = np.arange(n // 4, dtype=np.uint64)
            w = philox.philox4x32(blocks, 0, 0, 0, seed & 0xFFFFFFFF, seed >> 32)
            want = np.stack(w, axis=1).reshape(-1)
            # the order in which the library lays blocks out in memory is its own business: compare as sets of blocks
            got_blocks = {tuple(int(v) for v in got[i:i + 4]) for i in range(0, n, 4)}
            want_blocks = {tuple(int(v) for v in want[i:i + 4]) for i in range(0, n, 4)}
            assert got_blocks == want_blocks
    finally:
        rr.rocrand_destroy_generator(gen)
