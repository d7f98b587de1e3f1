"""CPU checks of the test-side helpers that GPU parity tests rely on."""
import numpy as np
import torch

from paper_1711_04325_amd import synth
from tests.gpu_util import bf16_round


def test_bf16_rounding_helper():
    """The test-side rounding against hand-worked cases: ties go to the even 8-bit significand."""
    a = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -8 + 2.0 ** -20), 3.140625, 0.0],
                 dtype=np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -7), 3.140625, 0.0])
    np.testing.assert_array_equal(bf16_round(a), want)
    t = torch.from_numpy(synth.normal(synth.rng(5), 4096).astype(np.float32))
    np.testing.assert_array_equal(bf16_round(t.numpy()), t.to(torch.bfloat16).to(torch.float64).numpy())
