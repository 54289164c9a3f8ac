"""The comparator itself: it must accept legitimate near-tie permutations and reject real errors."""
import numpy as np
import pytest

from compare import IP, L2, check_row, check_row_ids_only


def test_exact_match_passes():
    ids_o = np.array([5, 3, 9, 1, 7]); val_o = np.array([0.9, 0.8, 0.7, 0.6, 0.5])
    assert check_row(ids_o[:3], val_o[:3], ids_o, val_o, 3, 1e-4, 1.0, IP) == 3


def test_swap_inside_tie_group_passes_and_outside_fails():
    ids_o = np.array([5, 3, 9, 1, 7]); val_o = np.array([0.9, 0.80001, 0.8, 0.6, 0.5])
    check_row([5, 9, 3], [0.9, 0.800004, 0.800003], ids_o, val_o, 3, 1e-4, 1.0, IP)
    with pytest.raises(AssertionError):
        check_row([3, 5, 9], [0.9, 0.8, 0.8], ids_o, val_o, 3, 1e-4, 1.0, IP)


def test_boundary_group_may_contribute_any_member():
    ids_o = np.array([5, 3, 9, 1, 7]); val_o = np.array([0.1, 0.2, 0.30000, 0.30001, 0.5])
    check_row([5, 3, 1], [0.1, 0.2, 0.3], ids_o, val_o, 3, 1e-4, 1.0, L2)
    with pytest.raises(AssertionError):
        check_row([5, 3, 7], [0.1, 0.2, 0.3], ids_o, val_o, 3, 1e-4, 1.0, L2)


def test_value_error_and_bad_padding_fail():
    ids_o = np.array([5, 3, -1, -1]); val_o = np.array([0.1, 0.2, np.inf, np.inf])
    check_row([5, 3, -1], [0.1, 0.2, np.inf], ids_o, val_o, 3, 1e-4, 1.0, L2)
    with pytest.raises(AssertionError):
        check_row([5, 3, -1], [0.1, 0.2005, np.inf], ids_o, val_o, 3, 1e-4, 1.0, L2)
    with pytest.raises(AssertionError):
        check_row([5, 3, 0], [0.1, 0.2, np.inf], ids_o, val_o, 3, 1e-4, 1.0, L2)
    with pytest.raises(AssertionError):
        check_row([5, 3, -1], [0.1, 0.2, -np.inf], ids_o, val_o, 3, 1e-4, 1.0, L2)


def test_equal_values_need_ascending_ids():
    ids_o = np.array([2, 8, 4]); val_o = np.array([1.0, 1.0, 0.5])
    check_row([2, 8], [1.0, 1.0], ids_o, val_o, 2, 1e-4, 1.0, IP)
    with pytest.raises(AssertionError):
        check_row([8, 2], [1.0, 1.0], ids_o, val_o, 2, 1e-4, 1.0, IP)


def test_missing_id_needs_a_longer_oracle_row():
    ids_o = np.array([5, 3, 9]); val_o = np.array([0.5, 0.40001, 0.4])
    with pytest.raises(AssertionError, match="raise kx"):
        check_row([5, 77], [0.5, 0.4], ids_o, val_o, 2, 1e-4, 1.0, IP)
    with pytest.raises(AssertionError, match="not among"):
        check_row([77, 3], [0.5, 0.4], ids_o, val_o, 2, 1e-4, 1.0, IP)


def test_ids_only_variant():
    ids_o = np.array([4, 1, 6, 2]); val_o = np.array([9.0, 8.0, 7.9995, 3.0])
    check_row_ids_only(np.array([4, 6]), ids_o, val_o, 2, 1e-4, 1.0)
    with pytest.raises(AssertionError):
        check_row_ids_only(np.array([4, 2]), ids_o, val_o, 2, 1e-4, 1.0)
