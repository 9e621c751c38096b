"""The error measures of oracle/parity.py on arrays whose answers are known by hand."""
import numpy as np

from oracle.parity import G_FLOOR, gradient_errors


def test_every_sequence_is_measured_on_its_own_scale():
    cu = np.array([0, 2, 2, 5], dtype=np.int32)           # lengths 2, 0, 3
    want = np.zeros((5, 1, 2))
    want[:2] = 10.0                                        # a short sequence with large gradients
    want[2:] = 0.5                                         # a long one with small gradients
    got = want.copy()
    got[4, 0, 1] += 0.05                                   # 10 % of the long sequence's scale, 0.5 % of the batch's
    rel, fro = gradient_errors(got, want, cu)
    assert abs(rel - 0.1) < 1e-12
    assert abs(fro - 0.05 / np.linalg.norm(want)) < 1e-12
    got = want.copy()
    got[0, 0, 0] -= 1.0
    assert abs(gradient_errors(got, want, cu)[0] - 0.1) < 1e-12


def test_vanishing_gradients_are_measured_against_the_floor():
    cu = np.array([0, 1], dtype=np.int32)
    want = np.zeros((1, 2, 4))
    got = want + 0.5 * G_FLOOR * 1e-2
    rel, fro = gradient_errors(got, want, cu)
    assert abs(rel - 0.5e-2) < 1e-12 and fro > 1.0       # Frobenius ratio of a zero reference is meaningless
    assert gradient_errors(np.zeros((0, 1, 4)), np.zeros((0, 1, 4)), np.array([0], dtype=np.int32)) == (0.0, 0.0)
