"""Pins for the sparse x sparse oracle (oracle/spgemm.py)."""
import numpy as np

import oracle


def _merge_product(A, gamma, B, omega, k):
    """Section III-A as printed: per output block, walk the two sorted lists of kept block
    columns and multiply where both have the column."""
    Ra, N = gamma.shape
    Rb = omega.shape[0]
    C = np.zeros((Ra * k, Rb * k))
    count = 0
    for i in range(Ra):
        la = [c for c in range(N) if gamma[i, c]]
        for j in range(Rb):
            lb = [c for c in range(N) if omega[j, c]]
            x = y = 0
            while x < len(la) and y < len(lb):          # merge of two ascending lists
                if la[x] < lb[y]:
                    x += 1
                elif la[x] > lb[y]:
                    y += 1
                else:
                    c = la[x]
                    C[i * k:(i + 1) * k, j * k:(j + 1) * k] += (
                        A[i * k:(i + 1) * k, c * k:(c + 1) * k] @ B[j * k:(j + 1) * k, c * k:(c + 1) * k].T)
                    count += 1
                    x += 1
                    y += 1
    return C, count


def test_against_merge_of_sorted_lists():
    rng = np.random.default_rng(0)
    for k, Ra, Rb, N in ((8, 5, 4, 7), (1, 9, 6, 11), (4, 3, 3, 5)):
        A = rng.standard_normal((Ra * k, N * k))
        B = rng.standard_normal((Rb * k, N * k))
        gamma = (rng.random((Ra, N)) < 0.5).astype(np.uint8)
        omega = (rng.random((Rb, N)) < 0.5).astype(np.uint8)
        want, count = _merge_product(A, gamma, B, omega, k)
        got = oracle.spgemm_nt(A, gamma, B, omega, k)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
        assert oracle.matching_block_products(gamma, omega) == count


def test_hand_sized_case():
    # k = 1, N = 2: A = [[1, 2], [3, 4]] with gamma = [[1, 0], [1, 1]];
    # B = [[5, 6], [7, 8]] with omega = [[0, 1], [1, 1]]
    A = np.array([[1.0, 2.0], [3.0, 4.0]])
    B = np.array([[5.0, 6.0], [7.0, 8.0]])
    gamma = np.array([[1, 0], [1, 1]], dtype=np.uint8)
    omega = np.array([[0, 1], [1, 1]], dtype=np.uint8)
    # masked A = [[1, 0], [3, 4]], masked B = [[0, 6], [7, 8]]; C = Am Bm^t
    want = np.array([[1 * 0 + 0 * 6, 1 * 7 + 0 * 8], [3 * 0 + 4 * 6, 3 * 7 + 4 * 8]], dtype=float)
    assert (oracle.spgemm_nt(A, gamma, B, omega, 1) == want).all()
    assert oracle.matching_block_products(gamma, omega) == 0 + 1 + 1 + 2
    # masked-out contents are never used
    A2 = A.copy()
    A2[0, 1] = 1e30
    assert (oracle.spgemm_nt(A2, gamma, B, omega, 1) == want).all()
