"""Pins for oracle/memory_model.py: the operator identities Sec. 2 and App. A
state, checked on explicit matrices (adjoint == transpose under the Euclidean
inner product)."""
import numpy as np

from oracle import memory_model as mm

M = 7
A_IDX, B_IDX = [0, 2], [4, 5]


def test_allocation_adjoint_is_deallocation():
    # Sec. 2 Allocation: A_b^* = D_b and D_b^* = A_b
    A = mm.allocate(4, 3)
    D = mm.deallocate(7, 3)
    assert np.array_equal(A.T, D)
    x = np.arange(1.0, 5.0)
    assert np.array_equal(A @ x, [1, 2, 3, 4, 0, 0, 0])
    assert np.array_equal(D @ np.arange(7.0), [0, 1, 2, 3])


def test_clear_is_self_adjoint_and_idempotent():
    K = mm.clear(M, B_IDX)
    assert np.array_equal(K, K.T)
    assert np.array_equal(K @ K, K)
    x = np.arange(1.0, M + 1)
    out = K @ x
    assert out[4] == 0 and out[5] == 0 and out[0] == 1 and out[6] == 7


def test_add_adjoint_is_reverse_add():
    # Sec. 2 Add: S*_{a->b} = S_{b->a}
    S = mm.add(M, A_IDX, B_IDX)
    assert np.array_equal(S.T, mm.add(M, B_IDX, A_IDX))
    x = np.arange(1.0, M + 1)
    out = S @ x
    assert out[4] == x[4] + x[0] and out[5] == x[5] + x[2] and out[0] == x[0]


def test_in_place_copy_and_adjoint():
    # Sec. 2 Copy + App. A: C = S K_b, C* = K_b S_{b->a}
    C = mm.copy_in_place(M, A_IDX, B_IDX)
    x = np.arange(1.0, M + 1)
    out = C @ x
    assert out[4] == x[0] and out[5] == x[2]          # old x_b is gone
    assert np.array_equal(C.T, mm.copy_in_place_adjoint(M, A_IDX, B_IDX))
    # explicit block form of App. A: [[I, O], [I, O]]
    C2 = mm.copy_in_place(2, [0], [1])
    assert np.array_equal(C2, [[1, 0], [1, 0]])


def test_out_of_place_copy_and_adjoint():
    C = mm.copy_out_of_place(3, [0, 1, 2])
    assert np.array_equal(C, np.vstack([np.eye(3), np.eye(3)]))    # App. A: [I; I]
    assert np.array_equal(C.T, mm.copy_out_of_place_adjoint(3, [0, 1, 2]))


def test_move_adjoint_is_reverse_move():
    # Sec. 2 Move: M*_{a->b} = M_{b->a}
    Mv = mm.move_in_place(M, A_IDX, B_IDX)
    assert np.array_equal(Mv.T, mm.move_in_place_adjoint(M, A_IDX, B_IDX))
    assert np.array_equal(Mv.T, mm.move_in_place(M, B_IDX, A_IDX))
    assert np.array_equal(mm.move_in_place(2, [0], [1]), [[0, 0], [1, 0]])   # App. A
