"""The table checksum used for the stored full-size results: the numpy form under oracle/
and its torch retyping in the GPU parity tests must be the same function."""
import numpy as np
import torch

from oracle.checksum import table_checksum
from test_gpu_parity import torch_checksum


def test_hand_computed_values():
    # one cell a_0 = 0: (0 + 3) * ((0 * G + 0x7F4A7C15) | 1)
    assert table_checksum(np.array([0], np.int32)) == 3 * 0x7F4A7C15
    # a = [-1, 5]: 2 * w_0 + 8 * w_1 with w_1 = (G + 0x7F4A7C15) | 1, all mod 2^64
    w1 = ((0x9E3779B97F4A7C15 + 0x7F4A7C15) % (1 << 64)) | 1
    assert table_checksum(np.array([-1, 5], np.int64)) == (2 * 0x7F4A7C15 + 8 * w1) % (1 << 64)


def test_numpy_and_torch_forms_agree_and_detect_changes():
    rng = np.random.default_rng(5)
    for dtype, shape in ((np.int32, (7, 301, 13)), (np.int64, (1000, 33)), (np.int32, (1, 1))):
        a = rng.integers(-1, 1 << 20, size=shape).astype(dtype)
        if dtype == np.int64:
            a[::7] = 1 << 62
        ref = table_checksum(a)
        assert torch_checksum(torch.from_numpy(a)) == ref
        b = a.copy()
        b.flat[b.size // 2] += 1
        assert table_checksum(b) != ref
        if a.size > 2:
            c = a.copy().reshape(-1)
            c[[0, -1]] = c[[-1, 0]]
            if c[0] != c[-1]:
                assert table_checksum(c) != ref
    # chunked evaluation: a first_index continues the flat index
    a = rng.integers(0, 99, size=5000).astype(np.int32)
    whole = table_checksum(a)
    parts = (table_checksum(a[:1234]) + table_checksum(a[1234:], first_index=1234)) % (1 << 64)
    assert whole == parts
