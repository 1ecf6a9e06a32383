"""The comparison rules of the GPU tests themselves, exercised on the CPU with planted cases."""
import numpy as np
import pytest

import oracle
from gpu_util import assert_bf16_roundings


def test_bf16_rounding_rule_accepts_only_boundary_straddles():
    # 1 + 2^-8 lies exactly between the bfloat16 numbers 1 and 1 + 2^-7
    pre = np.array([1.00390625, 2.5, -3.0], np.float32)
    stored = oracle.round_bf16(pre.copy())
    assert_bf16_roundings(stored, pre)
    other = stored.copy()
    other[0] = 1.0078125 if stored[0] == 1.0 else 1.0
    assert_bf16_roundings(other, pre)                     # the other neighbour of a value on the boundary
    off = stored.copy()
    off[1] = 2.515625                                     # one step away although 2.5 is exactly representable
    with pytest.raises(AssertionError):
        assert_bf16_roundings(off, pre)
    far = stored.copy()
    far[0] = 1.015625                                     # two steps away
    with pytest.raises(AssertionError):
        assert_bf16_roundings(far, pre)
    # near zero the float32 tolerance spans several bfloat16 steps: anything inside it is a legitimate rounding
    assert_bf16_roundings(np.array([0.0, 7.5e-6], np.float32), np.array([3e-6, 0.0], np.float32))
    with pytest.raises(AssertionError):
        assert_bf16_roundings(np.array([3e-5], np.float32), np.array([0.0], np.float32))
