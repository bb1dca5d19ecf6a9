"""Pins for the gradient-sum + solver-update oracle (Eq. 1 plus history terms).

The float build is the bit-exact specification of the GPU kernel, so it is pinned
against numpy float32 scalar arithmetic (each operation rounded to float32),
closed forms that are exact in floating point, and the invariants of Eq. 1.
"""
import numpy as np
import pytest

F32 = np.float32


def _mk(rng, n, K, v_zero=False):
    w = (rng.standard_normal(n) * 1e-2).astype(F32)
    v = np.zeros(n, F32) if v_zero else (rng.standard_normal(n) * 1e-4).astype(F32)
    g = (rng.standard_normal(n) * 1e-3).astype(F32)
    peers = [(rng.standard_normal(n) * 1e-3).astype(F32) for _ in range(K)]
    return w, v, g, peers


def _numpy_f32_steps(w, v, g, peers, lr, mu, wd, gs=1.0):
    """Array-at-a-time float32 arithmetic: numpy rounds every ufunc result to float32."""
    lr, mu, wd, gs = F32(lr), F32(mu), F32(wd), F32(gs)
    s = g.copy()
    for p in peers:
        s = s + p
    if gs != F32(1):
        s = s * gs
    d = s + wd * w
    vn = mu * v + lr * d
    return w - vn, vn


@pytest.mark.parametrize("K", [0, 1, 4, 8, 16])
@pytest.mark.parametrize("gs", [1.0, 0.2])
def test_bit_exact_vs_numpy_float32(orc32, K, gs):
    rng = np.random.default_rng(100 + K)
    w, v, g, peers = _mk(rng, 10007, K)
    ew, ev = _numpy_f32_steps(w, v, g, peers, 0.01, 0.9, 5e-4, gs)
    orc32.grad_reduce_sgd(w, v, g, peers, 0.01, 0.9, 5e-4, gs)
    assert w.tobytes() == ew.tobytes() and v.tobytes() == ev.tobytes()


def test_eq1_without_history_terms(orc32):
    """mu = 0, wd = 0  =>  w' = w - lr * (g_0 + ... + g_K), summed left to right."""
    rng = np.random.default_rng(1)
    w, v, g, peers = _mk(rng, 5000, 4)
    w0 = w.copy()
    orc32.grad_reduce_sgd(w, v, g, peers, 0.01, 0.0, 0.0)
    s = g.copy()
    for p in peers:
        s = s + p
    step = F32(0.01) * s
    assert np.array_equal(v, step + F32(0) * F32(0)) and np.array_equal(w, w0 - step)


def test_order_is_left_to_right_local_first(orc32):
    """(big + small) + (-big) differs from (big + (-big)) + small in float32."""
    n = 8
    g = np.full(n, 1e8, F32)
    peers = [np.full(n, 1.0, F32), np.full(n, -1e8, F32)]
    w, v = np.zeros(n, F32), np.zeros(n, F32)
    orc32.grad_reduce_sgd(w, v, g, peers, 1.0, 0.0, 0.0)
    assert np.all(v == F32(0.0))          # 1e8 + 1 rounds back to 1e8
    w, v = np.zeros(n, F32), np.zeros(n, F32)
    orc32.grad_reduce_sgd(w, v, g, peers[::-1], 1.0, 0.0, 0.0)
    assert np.all(v == F32(1.0))


@pytest.mark.parametrize("K", [4, 8, 16])
def test_identical_buffers_sum_to_multiple(orc32, K):
    """Inputs with at most 12 significant bits: every partial sum is exact, so the sum of
    K+1 copies is (K+1)*g bit for bit."""
    rng = np.random.default_rng(2)
    g = (rng.integers(-2048, 2048, 4096) / 1024.0).astype(F32)
    w, v = np.zeros(4096, F32), np.zeros(4096, F32)
    orc32.grad_reduce_sgd(w, v, g, [g.copy() for _ in range(K)], 1.0, 0.0, 0.0)
    assert np.array_equal(v, F32(K + 1) * g) and np.array_equal(w, -(F32(K + 1) * g))


def test_five_identical_arbitrary_buffers(orc32):
    """For m <= 5 the sequential sum of m equal floats is exactly fl(m*g) for any g."""
    rng = np.random.default_rng(3)
    g = rng.standard_normal(50000).astype(F32)
    w, v = np.zeros(g.size, F32), np.zeros(g.size, F32)
    orc32.grad_reduce_sgd(w, v, g, [g.copy() for _ in range(4)], 1.0, 0.0, 0.0)
    assert np.array_equal(v, F32(5) * g)


def test_zero_learning_rate(orc32):
    rng = np.random.default_rng(4)
    w, v, g, peers = _mk(rng, 3000, 4, v_zero=True)
    w0 = w.copy()
    orc32.grad_reduce_sgd(w, v, g, peers, 0.0, 0.9, 5e-4)
    assert w.tobytes() == w0.tobytes() and not v.any()
    # with history the solver form still moves: w' = w - mu*v, v' = mu*v
    w, v, g, peers = _mk(rng, 3000, 4)
    w0, v0 = w.copy(), v.copy()
    orc32.grad_reduce_sgd(w, v, g, peers, 0.0, 0.9, 5e-4)
    assert np.array_equal(v, F32(0.9) * v0) and np.array_equal(w, w0 - F32(0.9) * v0)


def test_single_worker_plain_sgd(orc32):
    rng = np.random.default_rng(5)
    w, v, g, _ = _mk(rng, 3000, 0, v_zero=True)
    w0 = w.copy()
    orc32.grad_reduce_sgd(w, v, g, [], 1.0, 0.0, 0.0)
    assert np.array_equal(w, w0 - g) and np.array_equal(v, g)


def test_weight_decay_pulls_towards_zero(orc32):
    w = np.array([2.0, -4.0], F32)
    v = np.zeros(2, F32)
    orc32.grad_reduce_sgd(w, v, np.zeros(2, F32), [], 0.5, 0.0, 0.25)
    assert np.array_equal(v, [0.25, -0.5]) and np.array_equal(w, [1.75, -3.5])


def test_two_steps_momentum_closed_form(orc64):
    """Constant gradient, wd = 0: v2 = lr*g*(1+mu), w2 = w0 - lr*g*(2+mu)."""
    g = np.array([0.5, -1.5, 3.0])
    w, v = np.array([1.0, 2.0, 3.0]), np.zeros(3)
    for _ in range(2):
        orc64.grad_reduce_sgd(w, v, g, [], 0.1, 0.9, 0.0)
    np.testing.assert_allclose(v, 0.1 * g * 1.9, rtol=1e-15)
    np.testing.assert_allclose(w, np.array([1.0, 2.0, 3.0]) - 0.1 * g * 2.9, rtol=1e-15)


def test_grad_scale_gives_the_mean(orc32):
    g = np.array([1.0, 2.0, -3.0], F32)
    w, v = np.zeros(3, F32), np.zeros(3, F32)
    orc32.grad_reduce_sgd(w, v, g, [g.copy()] * 3, 1.0, 0.0, 0.0, 0.25)
    assert np.array_equal(v, g)


def test_denormals_and_nonfinite_propagate(orc32):
    tiny = np.float32(1e-45)
    w, v = np.zeros(3, F32), np.zeros(3, F32)
    g = np.array([tiny, np.inf, np.nan], F32)
    orc32.grad_reduce_sgd(w, v, g, [np.array([tiny, 0, 0], F32)], 1.0, 0.0, 0.0)
    assert v[0] == np.float32(2) * tiny and v[0] != 0 and np.isinf(v[1]) and np.isnan(v[2])


# ---- binomial-tree association (section 3.2 "Reduction of the Gradient") -------------------------

def _tree_by_rounds(bufs):
    """A second formulation of the reduction tree, by message rounds: in the round of distance d
    every rank whose lowest set bit is d sends its running sum to rank r - d, which adds it.
    float32 arrays, each addition rounded once.  Returns (sum held by rank 0, number of rounds,
    list of (sender, receiver))."""
    acc = [b.astype(F32).copy() for b in bufs]
    m, d, rounds, msgs = len(acc), 1, 0, []
    while d < m:
        for r in range(d, m, 2 * d):
            acc[r - d] = acc[r - d] + acc[r]
            msgs.append((r, r - d))
        d *= 2
        rounds += 1
    return acc[0], rounds, msgs


def _tree_sum_oracle(orc32, bufs):
    n = bufs[0].size
    w, v = np.zeros(n, F32), np.zeros(n, F32)
    orc32.grad_reduce_sgd(w, v, bufs[0], bufs[1:], 1.0, 0.0, 0.0, order="tree")
    assert np.array_equal(w, -v)
    return v


@pytest.mark.parametrize("K", list(range(0, 17)) + [23, 31, 32, 63])
def test_tree_matches_message_rounds(orc32, K):
    rng = np.random.default_rng(700 + K)
    bufs = [rng.standard_normal(3001).astype(F32) for _ in range(K + 1)]
    ref, rounds, msgs = _tree_by_rounds(bufs)
    assert np.array_equal(_tree_sum_oracle(orc32, bufs), ref)
    # shape of the tree: every rank but the master sends exactly once, to a lower rank,
    # and the depth is ceil(log2(K + 1))
    assert sorted(s for s, _ in msgs) == list(range(1, K + 1)) and all(r < s for s, r in msgs)
    assert rounds == int(np.ceil(np.log2(K + 1)))


def test_tree_rounding_cases_worked_by_hand(orc32):
    """u = 2^-23 is one unit in the last place of 1.0; ties round to even.
    Four ranks (1, u/2, u/2, u/2): the tree forms (1 + u/2) + (u/2 + u/2) = 1 + u, while left to
    right every u/2 is lost.  Eight ranks (1, then seven u/2): ((1+u/2) + u) + 2u = 1 + 3u."""
    u = F32(2.0 ** -23)
    one = np.ones(4, F32)
    half = np.full(4, u / F32(2), F32)
    assert np.all(_tree_sum_oracle(orc32, [one, half, half, half]) == F32(1) + u)
    w, v = np.zeros(4, F32), np.zeros(4, F32)
    orc32.grad_reduce_sgd(w, v, one, [half] * 3, 1.0, 0.0, 0.0)
    assert np.all(v == F32(1))
    assert np.all(_tree_sum_oracle(orc32, [one] + [half] * 7) == F32(1) + F32(3) * u)


def test_tree_adds_the_nearest_sender_first(orc32):
    """Three ranks (1, u/2, 3u/4): (1 + u/2) + 3u/4 = 1 + u, but (1 + 3u/4) + u/2 = 1 + 2u."""
    u = F32(2.0 ** -23)
    a, b, c = np.ones(2, F32), np.full(2, u * F32(0.5), F32), np.full(2, u * F32(0.75), F32)
    assert np.all(_tree_sum_oracle(orc32, [a, b, c]) == F32(1) + u)
    assert np.all(_tree_sum_oracle(orc32, [a, c, b]) == F32(1) + F32(2) * u)


@pytest.mark.parametrize("K", [0, 1, 2])
def test_tree_equals_left_to_right_up_to_three_ranks(orc32, K):
    rng = np.random.default_rng(710 + K)
    w, v, g, peers = _mk(rng, 4099, K)
    w2, v2 = w.copy(), v.copy()
    orc32.grad_reduce_sgd(w, v, g, peers, 0.01, 0.9, 5e-4, 0.5)
    orc32.grad_reduce_sgd(w2, v2, g, peers, 0.01, 0.9, 5e-4, 0.5, order="tree")
    assert w.tobytes() == w2.tobytes() and v.tobytes() == v2.tobytes()


@pytest.mark.parametrize("K", [4, 8, 16])
def test_tree_history_terms_and_reassociation_bound(orc32, K):
    """The steps after the sum are those of the sequential form (checked through numpy float32 on
    the message-round sum), and the two associations differ by at most K ulp of the largest
    partial sum."""
    rng = np.random.default_rng(720 + K)
    w, v, g, peers = _mk(rng, 20011, K)
    s, _, _ = _tree_by_rounds([g] + peers)
    lr, mu, wd, gs = F32(0.01), F32(0.9), F32(5e-4), F32(0.25)
    vn = mu * v + lr * (s * gs + wd * w)
    ew = w - vn
    w2, v2 = w.copy(), v.copy()
    orc32.grad_reduce_sgd(w2, v2, g, peers, 0.01, 0.9, 5e-4, 0.25, order="tree")
    assert w2.tobytes() == ew.tobytes() and v2.tobytes() == vn.tobytes()
    seq = g.copy()
    for p in peers:
        seq = seq + p
    bound = K * np.spacing(np.abs(np.stack([g] + peers)).sum(0).astype(F32))
    assert np.all(np.abs(seq.astype(np.float64) - s.astype(np.float64)) <= bound)
    assert np.any(seq != s)


@pytest.mark.parametrize("K", [4, 8, 16])
def test_tree_exact_inputs_give_the_exact_sum(orc32, K):
    rng = np.random.default_rng(730 + K)
    bufs = [(rng.integers(-2048, 2048, 4096) / 1024.0).astype(F32) for _ in range(K + 1)]
    exact = np.sum(np.stack(bufs).astype(np.float64), 0)
    assert np.array_equal(_tree_sum_oracle(orc32, bufs).astype(np.float64), exact)


def test_tree_rounding_cases_from_the_fixture(orc32):
    """tests/golden/tree_sum_rounding.txt: sums worked by hand, tree order and left to right."""
    import os
    u = F32(2.0 ** -23)
    path = os.path.join(os.path.dirname(__file__), "golden", "tree_sum_rounding.txt")
    cases = 0
    for line in open(path):
        if not line.startswith("ranks"):
            continue
        tok = line.split()
        vals = tok[1:tok.index("tree")]
        tree, seq = float(tok[tok.index("tree") + 1]), float(tok[tok.index("seq") + 1])
        bufs = [np.full(3, F32(1) if v == "1" and i == 0 else F32(float(v)) * u, F32) for i, v in enumerate(vals)]
        assert np.all(_tree_sum_oracle(orc32, bufs) == F32(1) + F32(tree) * u), line
        w, v = np.zeros(3, F32), np.zeros(3, F32)
        orc32.grad_reduce_sgd(w, v, bufs[0], bufs[1:], 1.0, 0.0, 0.0)
        assert np.all(v == F32(1) + F32(seq) * u), line
        cases += 1
    assert cases == 5
