"""Sec. 2 "Linear algebraic memory model": the primitive memory operations
written out as the block matrices the paper gives for them.

A "memory" is a vector of length m split into named, disjoint index subsets
(a, b, ...).  Every operator below returns a dense fp64 matrix acting on such
a vector, so that adjoints can be checked as plain transposes under the
Euclidean inner product (Sec. 2, first two displayed equations).

Test infrastructure only (see the package docstring).
"""
import numpy as np


def _eye_on(idx, m):
    """m x m matrix that is the identity on index set idx and zero elsewhere."""
    mat = np.zeros((m, m))
    for i in idx:
        mat[i, i] = 1.0
    return mat


def allocate(m, n_new):
    """A_b (Sec. 2, Allocation): [I_a; O_b] -- maps F^m to F^(m+n_new) and
    brings n_new zero-valued cells into scope after the existing ones."""
    return np.vstack([np.eye(m), np.zeros((n_new, m))])


def deallocate(m, n_drop):
    """D_b (Sec. 2, Allocation): [I_a  O_b] -- drops the trailing n_drop cells.
    The paper states D_b = A_b^* and D_b^* = A_b."""
    return np.hstack([np.eye(m - n_drop), np.zeros((m - n_drop, n_drop))])


def clear(m, b):
    """K_b (Sec. 2, Clear): identity off b, zero on b.  Self-adjoint."""
    keep = [i for i in range(m) if i not in set(b)]
    return _eye_on(keep, m)


def add(m, a, b):
    """S_{a->b} (Sec. 2, Add): x_b <- x_a + x_b, x_a unchanged.
    a and b are equal-length index lists; a[i] is added onto b[i]."""
    assert len(a) == len(b)
    mat = np.eye(m)
    for ia, ib in zip(a, b):
        mat[ib, ia] += 1.0
    return mat


def copy_in_place(m, a, b):
    """C_{a->b} = S_{a->b} K_b (Sec. 2, Copy, in-place form)."""
    return add(m, a, b) @ clear(m, b)


def copy_in_place_adjoint(m, a, b):
    """C*_{a->b} = K_b S_{b->a} (Sec. 2, Copy, in-place form)."""
    return clear(m, b) @ add(m, b, a)


def copy_out_of_place(m, a):
    """C_{a->b} = S_{a->b} A_b (Sec. 2, Copy, out-of-place form): b is a fresh
    block of len(a) cells appended after the m existing ones."""
    nb = len(a)
    b = list(range(m, m + nb))
    return add(m + nb, a, b) @ allocate(m, nb)


def copy_out_of_place_adjoint(m, a):
    """C*_{a->b} = D_b S_{b->a} (Sec. 2, Copy, out-of-place form)."""
    nb = len(a)
    b = list(range(m, m + nb))
    return deallocate(m + nb, nb) @ add(m + nb, b, a)


def move_in_place(m, a, b):
    """M_{a->b} = K_a S_{a->b} K_b (Sec. 2, Move, in-place form)."""
    return clear(m, a) @ add(m, a, b) @ clear(m, b)


def move_in_place_adjoint(m, a, b):
    """M*_{a->b} = K_b S_{b->a} K_a = M_{b->a} (Sec. 2, Move)."""
    return clear(m, b) @ add(m, b, a) @ clear(m, a)
