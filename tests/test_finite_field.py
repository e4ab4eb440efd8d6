"""The paper's random tests over finite fields, applied to the one rewrite this library rests on.

CPU part (no GPU): the oracle's modular evaluation is pinned to field facts (Fermat inverses, roots
that square back, a hand case) and the two graph forms agree on random inputs, while a planted wrong
rewrite is caught.  GPU part: the integer kernel equals the oracle bit for bit, in both forms.
"""
import numpy as np
import pytest

import oracle

P, Q = 227, 113          # the primes the paper's implementation uses (q divides p - 1)


def _rand(M, K, N, p, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, p, (M, K)), rng.integers(0, p, K), rng.integers(0, p, (K, N))


def test_canonical_root():
    for p in (P, Q, 7):
        residues = {y * y % p for y in range(p)}
        nonres = next(v for v in range(2, p) if v not in residues)
        for x in range(p):
            r = oracle.ff_sqrt(x, p)
            if x in residues:
                assert r * r % p == x and all(y * y % p != x for y in range(r))
            else:
                assert r * r % p == x * nonres % p
            assert (r == 0) == (x == 0)


def test_hand_case_mod_7():
    """X = [[1, 2]], g = [1, 1], W = [[1], [1]], p = 7: A = 5, 1/K = 4, mean = 6 (a non-residue of 7:
    squares are 0, 1, 2, 4; least non-residue 3, 6*3 = 4, root 2), 1/2 = 4; (1 + 2) * 4 = 12 = 5."""
    for reordered in (False, True):
        Y = oracle.ff_rmsnorm_linear([[1, 2]], [1, 1], [[1], [1]], 7, reordered)
        assert Y.tolist() == [[5]]


@pytest.mark.parametrize("p", [P, Q, 7, 32749])
def test_rewrite_holds_over_the_field(p):
    """Division distributes over the sum in any field: the two forms agree exactly on random inputs."""
    for seed in range(4):
        X, g, W = _rand(5, 24, 9, p, 100 * p + seed)
        a = oracle.ff_rmsnorm_linear(X, g, W, p, False)
        b = oracle.ff_rmsnorm_linear(X, g, W, p, True)
        assert np.array_equal(a, b)
        assert a.min() >= 0 and a.max() < p


def test_a_wrong_rewrite_is_caught():
    """Dividing by the root of the sum of squares of X (.) g instead of X is NOT the same graph:
    the random test tells them apart at once (this is what the verifier is for)."""
    X, g, W = _rand(4, 16, 6, P, 7)
    good = oracle.ff_rmsnorm_linear(X, g, W, P, True)
    bad = oracle.ff_rmsnorm_linear(X * g % P, np.ones_like(g), W, P, True)
    assert not np.array_equal(good, bad)


def test_zero_mean_square_row_is_zero():
    X = np.zeros((1, 8), dtype=np.int64)
    g, W = np.ones(8, dtype=np.int64), np.ones((8, 3), dtype=np.int64)
    assert not oracle.ff_rmsnorm_linear(X, g, W, P, False).any()
    assert not oracle.ff_rmsnorm_linear(X, g, W, P, True).any()


@pytest.mark.gpu
@pytest.mark.parametrize("p", [P, Q, 7, 32749])
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (3, 17, 5), (8, 64, 300), (33, 100, 257)])
def test_gpu_field_block_is_bit_exact(p, M, K, N):
    import torch
    import paper_2405_05751_amd as rl
    if K % p == 0:
        pytest.skip("p divides K")
    X, g, W = _rand(M, K, N, p, 9000 + p + M + K + N)
    if M >= 3:
        X[1] = 0                                     # a row without an inverse root
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    outs = []
    for reordered in (False, True):
        Y = rl.rl_ff_rmsnorm_linear(dev(X), dev(g), dev(W), p, reordered)
        torch.cuda.synchronize()
        want = oracle.ff_rmsnorm_linear(X, g, W, p, reordered)
        assert np.array_equal(Y.cpu().numpy().astype(np.int64), want)
        outs.append(Y)
    assert torch.equal(outs[0], outs[1])             # the verification itself


@pytest.mark.gpu
def test_gpu_field_block_rejects_bad_primes():
    import torch
    import paper_2405_05751_amd as rl
    t = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
    g = torch.zeros(4, dtype=torch.int32, device="cuda")
    for bad in (1, 2, 4, 221, 40000):
        with pytest.raises(rl.RmsnlError):
            rl.rl_ff_rmsnorm_linear(t, g, t.t().contiguous(), bad, False)
    with pytest.raises(rl.RmsnlError):
        rl.rl_ff_rmsnorm_linear(torch.zeros((2, 7), dtype=torch.int32, device="cuda"),
                                torch.zeros(7, dtype=torch.int32, device="cuda"),
                                torch.zeros((7, 2), dtype=torch.int32, device="cuda"), 7, False)
