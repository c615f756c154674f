"""Pins for the spatial-row anchor oracle (CPU only).

The paper prints no numerical example of an anchor output.  What it fixes: the
number of computed queries per frame (k*W instead of H*W, Section 3.3) and the
skipped fraction 1 - k/H printed for each k in the supplement's anchor table;
with every row an anchor the scheme is plain dense attention; the scheme is
exact whenever the queries of a frame do not depend on the spatial row.  The
rest is pinned by a scalar-loop brute force, by hand-worked row maps and by
mutants that must fail.
"""
import math
import os

import numpy as np
import pytest

from oracle import sparse_attention
from oracle import anchor as A
from workloads import f32_to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bits(rng, shape, gain=1.0):
    return f32_to_bf16_bits((gain * rng.standard_normal(shape)).astype(np.float32))


def _f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _table():
    rows = []
    with open(os.path.join(GOLDEN, "anchor_table.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            k, ms, sp, pct = (x.strip() for x in line.split("|"))
            rows.append((int(k), float(ms), float(sp), float(pct)))
    return rows


def test_query_counts_match_the_papers_table():
    """Wan 480p geometry: k*W computed queries per frame, skipped fraction 1 - k/H."""
    F, Hs, Ws = 21, 30, 52
    N = F * Hs * Ws
    rows = _table()
    assert [r[0] for r in rows] == [30, 15, 10, 5, 4, 3, 2, 1]
    for k, _, _, pct in rows:
        q_index, src = A.anchor_token_maps(N, F, Hs, Ws, k)
        assert q_index.size == F * k * Ws
        assert abs(100.0 * (1 - q_index.size / N) - pct) < 0.05
        assert np.unique(q_index).size == q_index.size
        assert src.min() == 0 and src.max() == q_index.size - 1


def test_hand_worked_rows():
    # 6 rows, 2 anchors: segment centres 1.5 and 4.5 -> rows 1 and 4
    assert A.anchor_rows(6, 2).tolist() == [1, 4]
    assert A.nearest_anchor(6, 2).tolist() == [0, 0, 0, 1, 1, 1]
    # 7 rows, 3 anchors: centres 7/6, 21/6, 35/6 -> rows 1, 3, 5; rows 2 and 4 tie -> lower anchor
    assert A.anchor_rows(7, 3).tolist() == [1, 3, 5]
    assert A.nearest_anchor(7, 3).tolist() == [0, 0, 0, 1, 1, 2, 2]
    # the paper's setting: 30 rows, 5 anchors -> centres 3, 9, 15, 21, 27
    assert A.anchor_rows(30, 5).tolist() == [3, 9, 15, 21, 27]
    near = A.nearest_anchor(30, 5)
    assert near.tolist() == [0] * 7 + [1] * 6 + [2] * 6 + [3] * 6 + [4] * 5
    assert A.anchor_rows(30, 1).tolist() == [15]
    assert A.anchor_rows(30, 30).tolist() == list(range(30))
    assert A.nearest_anchor(30, 30).tolist() == list(range(30))


def test_hand_worked_token_maps():
    # 2 frames of 3 rows x 2 columns, one anchor (row 1), plus 2 tokens without a position
    q_index, src = A.anchor_token_maps(14, 2, 3, 2, 1)
    assert q_index.tolist() == [2, 3, 8, 9, 12, 13]
    assert src.tolist() == [0, 1, 0, 1, 0, 1, 2, 3, 2, 3, 2, 3, 4, 5]


@pytest.mark.parametrize("n_rows", [1, 2, 5, 7, 30, 45])
def test_anchor_rows_are_spread_evenly(n_rows):
    for k in range(1, n_rows + 1):
        a = A.anchor_rows(n_rows, k)
        assert (np.diff(a) > 0).all() and a[0] >= 0 and a[-1] < n_rows
        if k > 1:
            gaps = np.diff(a)
            assert gaps.max() - gaps.min() <= 1  # equally spaced up to integer rounding
        # symmetric margins up to rounding: first anchor vs rows after the last
        assert abs(int(a[0]) - int(n_rows - 1 - a[-1])) <= 1
        near = A.nearest_anchor(n_rows, k)
        for y in range(n_rows):
            d = np.abs(a - y)
            assert d[near[y]] == d.min()
            assert near[y] == int(np.flatnonzero(d == d.min())[0])


def _brute(q, k, v, F, Hs, Ws, kk, scale):
    """Scalar loops, written separately from the oracle: every token looks up
    its own anchor and runs its own softmax."""
    N, D = len(q), len(q[0])
    centres = [((2 * j + 1) * Hs) // (2 * kk) for j in range(kk)]
    out = [[0.0] * D for _ in range(N)]
    for t in range(N):
        if t < F * Hs * Ws:
            f, rem = divmod(t, Hs * Ws)
            y, x = divmod(rem, Ws)
            best = min(centres, key=lambda a: (abs(a - y), a))
            tq = (f * Hs + best) * Ws + x
        else:
            tq = t
        logits = [scale * sum(q[tq][d] * k[j][d] for d in range(D)) for j in range(N)]
        m = max(logits)
        e = [math.exp(s - m) for s in logits]
        z = sum(e)
        for d in range(D):
            out[t][d] = sum(e[j] * v[j][d] for j in range(N)) / z
    return np.array(out)


@pytest.mark.parametrize("F,Hs,Ws,k,extra", [(2, 3, 2, 1, 0), (2, 5, 3, 2, 3), (1, 4, 2, 4, 1), (3, 7, 1, 3, 0)])
def test_brute_force(F, Hs, Ws, k, extra):
    rng = np.random.default_rng(100 + F + Hs + Ws + k)
    N, D = F * Hs * Ws + extra, 4
    q, kk, v = (_bits(rng, (1, 2, N, D), 1.5) for _ in range(3))
    got = A.anchor_attention(q, kk, v, [1], F, Hs, Ws, k, 0.37)
    want = _brute(_f64(q[0, 1]).tolist(), _f64(kk[0, 1]).tolist(), _f64(v[0, 1]).tolist(), F, Hs, Ws, k, 0.37)
    np.testing.assert_allclose(got[0, 0], want, rtol=1e-12, atol=1e-13)


def test_every_row_an_anchor_is_dense_attention():
    rng = np.random.default_rng(7)
    F, Hs, Ws, extra, D = 2, 4, 5, 3, 8
    N = F * Hs * Ws + extra
    q, k, v = (_bits(rng, (2, 3, N, D)) for _ in range(3))
    got = A.anchor_attention(q, k, v, [2, 0], F, Hs, Ws, Hs, 0.3)
    dense = sparse_attention(q, k, v, np.ones((3, 1, 1), np.uint8), None, 0.3, N, N)
    np.testing.assert_allclose(got[:, 0], dense[:, 2], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(got[:, 1], dense[:, 0], rtol=1e-12, atol=1e-14)


def test_exact_when_queries_do_not_depend_on_the_row():
    """If q[f, y, x] is the same for every y, rows of a frame have identical
    attention (the premise of Section 3.3) and any k reproduces dense attention."""
    rng = np.random.default_rng(8)
    F, Hs, Ws, D = 3, 6, 4, 8
    N = F * Hs * Ws
    base = _bits(rng, (1, 1, F, 1, Ws, D))
    q = np.broadcast_to(base, (1, 1, F, Hs, Ws, D)).reshape(1, 1, N, D).copy()
    k, v = _bits(rng, (1, 1, N, D)), _bits(rng, (1, 1, N, D))
    dense = sparse_attention(q, k, v, np.ones((1, 1, 1), np.uint8), None, 0.5, N, N)
    for kk in (1, 2, 3, 6):
        got = A.anchor_attention(q, k, v, [0], F, Hs, Ws, kk, 0.5)
        np.testing.assert_allclose(got, dense, rtol=1e-12, atol=1e-14)


def test_constant_values_and_shared_outputs():
    rng = np.random.default_rng(9)
    F, Hs, Ws, extra, D, k = 2, 7, 3, 2, 4, 3
    N = F * Hs * Ws + extra
    q, kk = _bits(rng, (1, 1, N, D)), _bits(rng, (1, 1, N, D))
    c = _bits(rng, (D,))
    v = np.broadcast_to(c, (1, 1, N, D)).copy()
    out = A.anchor_attention(q, kk, v, [0], F, Hs, Ws, k, 1.0)
    np.testing.assert_allclose(out, np.broadcast_to(_f64(c), out.shape), rtol=1e-13)
    # rows sharing an anchor hold identical outputs; rows with different anchors differ
    v2 = _bits(rng, (1, 1, N, D))
    out = A.anchor_attention(q, kk, v2, [0], F, Hs, Ws, k, 1.0)[0, 0, : F * Hs * Ws].reshape(F, Hs, Ws, D)
    near = A.nearest_anchor(Hs, k)
    for y in range(Hs):
        assert (out[:, y] == out[:, A.anchor_rows(Hs, k)[near[y]]]).all()
    assert not (out[:, 0] == out[:, Hs - 1]).all()
    assert not (out[0] == out[1]).all()  # frames are not mixed up


def test_chunking_changes_nothing():
    rng = np.random.default_rng(10)
    q, k, v = (_bits(rng, (1, 1, 60, 8)) for _ in range(3))
    a = A.anchor_attention(q, k, v, [0], 2, 5, 6, 2, 0.4, chunk=7)
    b = A.anchor_attention(q, k, v, [0], 2, 5, 6, 2, 0.4, chunk=4096)
    assert (a == b).all()


# ---------------------------------------------------------------------------
# spatial similarity score (detection of repetitive heads)
# ---------------------------------------------------------------------------
def _score_brute(q, k, F, Hs, Ws, kk, scale):
    """Scalar loops over every (frame, row): flattened probability vectors built entry by entry."""
    N, D = len(k), len(k[0])
    centres = [((2 * j + 1) * Hs) // (2 * kk) for j in range(kk)]

    def probs(t):
        logits = [scale * sum(q[t][d] * k[j][d] for d in range(D)) for j in range(N)]
        m = max(logits)
        e = [math.exp(x - m) for x in logits]
        z = sum(e)
        return [x / z for x in e]

    total = 0.0
    for f in range(F):
        for i in range(Hs):
            a = min(centres, key=lambda c: (abs(c - i), c))
            u, w = [], []
            for x in range(Ws):
                u += probs((f * Hs + i) * Ws + x)
                w += probs((f * Hs + a) * Ws + x)
            dot = sum(p1 * p2 for p1, p2 in zip(u, w))
            total += dot / math.sqrt(sum(p * p for p in u) * sum(p * p for p in w))
    return total / (F * Hs)


@pytest.mark.parametrize("F,Hs,Ws,k,extra", [(2, 3, 2, 1, 0), (1, 5, 2, 2, 3), (2, 4, 1, 3, 1)])
def test_score_brute_force(F, Hs, Ws, k, extra):
    rng = np.random.default_rng(300 + F + Hs + Ws + k)
    N, D = F * Hs * Ws + extra, 4
    q, kk = _bits(rng, (1, 2, N, D), 1.5), _bits(rng, (1, 2, N, D), 1.5)
    got = A.spatial_similarity(q, kk, F, Hs, Ws, k, 0.6)
    for h in range(2):
        want = _score_brute(_f64(q[0, h]).tolist(), _f64(kk[0, h]).tolist(), F, Hs, Ws, k, 0.6)
        assert abs(got[0, h] - want) < 1e-12


def test_score_is_the_mean_of_its_rows():
    rng = np.random.default_rng(12)
    F, Hs, Ws, k, D = 2, 5, 3, 2, 4
    N = F * Hs * Ws + 2
    q, kk = _bits(rng, (1, 2, N, D), 1.5), _bits(rng, (1, 2, N, D), 1.5)
    full = A.spatial_similarity(q, kk, F, Hs, Ws, k, 0.6)
    for h in range(2):
        rows = A.spatial_similarity_rows(q, kk, F, Hs, Ws, k, 0.6, [(0, h, f, i) for f in range(F) for i in range(Hs)])
        assert abs(np.mean(rows) - full[0, h]) < 1e-14


def test_score_special_cases():
    rng = np.random.default_rng(11)
    F, Hs, Ws, D = 2, 6, 3, 8
    N = F * Hs * Ws + 4
    k = _bits(rng, (1, 1, N, D), 2.0)
    q = _bits(rng, (1, 1, N, D), 2.0)
    # every row an anchor: each row is compared with itself
    np.testing.assert_allclose(A.spatial_similarity(q, k, F, Hs, Ws, Hs, 0.5), 1.0, rtol=1e-14)
    # queries that do not depend on the spatial row: identical attention rows, score 1 for any k
    base = _bits(rng, (1, 1, F, 1, Ws, D))
    qv = np.broadcast_to(base, (1, 1, F, Hs, Ws, D)).reshape(1, 1, F * Hs * Ws, D)
    q_same = np.concatenate([qv, q[:, :, F * Hs * Ws :]], axis=2)
    for kk in (1, 2, 3):
        np.testing.assert_allclose(A.spatial_similarity(q_same, k, F, Hs, Ws, kk, 0.5), 1.0, rtol=1e-14)
    # generic queries: strictly between 0 and 1, and more anchors never lower the score here
    s1 = A.spatial_similarity(q, k, F, Hs, Ws, 1, 0.5)[0, 0]
    s3 = A.spatial_similarity(q, k, F, Hs, Ws, 3, 0.5)[0, 0]
    assert 0 < s1 < s3 < 1


def test_score_one_hot_attention_counts_matching_rows():
    """Huge logits make every query attend to exactly one key: a row's cosine
    with its anchor is the fraction of columns that pick the same key."""
    F, Hs, Ws, D = 1, 4, 2, 4
    N = F * Hs * Ws
    kf = np.zeros((N, D), np.float32)
    for j in range(4):
        kf[j, j] = 1.0  # keys 0..3 are the unit vectors; the rest are zero
    qf = np.zeros((N, D), np.float32)
    pick = {(0, 0): 0, (0, 1): 1, (1, 0): 0, (1, 1): 1, (2, 0): 0, (2, 1): 3, (3, 0): 2, (3, 1): 3}
    for (i, x), j in pick.items():
        qf[i * Ws + x, j] = 200.0
    q, k = f32_to_bf16_bits(qf[None, None]), f32_to_bf16_bits(kf[None, None])
    # one anchor (row 2, picks keys 0 and 3): rows 0, 1 share column 0 only -> 1/2; row 2 -> 1; row 3 shares column 1 -> 1/2
    np.testing.assert_allclose(A.spatial_similarity(q, k, F, Hs, Ws, 1, 1.0), (0.5 + 0.5 + 1 + 0.5) / 4, rtol=1e-12)


# ---------------------------------------------------------------------------
# mutants: plausible mistakes planted in a copy of the oracle must be caught
# ---------------------------------------------------------------------------
def _run_pins(mod):
    """True if every pin passes for the module-like object ``mod``."""
    try:
        assert mod.anchor_rows(7, 3).tolist() == [1, 3, 5]
        assert mod.nearest_anchor(7, 3).tolist() == [0, 0, 0, 1, 1, 2, 2]
        assert mod.anchor_rows(30, 5).tolist() == [3, 9, 15, 21, 27]
        q_index, src = mod.anchor_token_maps(14, 2, 3, 2, 1)
        assert q_index.tolist() == [2, 3, 8, 9, 12, 13]
        assert src.tolist() == [0, 1, 0, 1, 0, 1, 2, 3, 2, 3, 2, 3, 4, 5]
        rng = np.random.default_rng(3)
        F, Hs, Ws, k, extra, D = 2, 5, 3, 2, 3, 4
        N = F * Hs * Ws + extra
        q, kk, v = (_bits(rng, (1, 1, N, D), 1.5) for _ in range(3))
        got = mod.anchor_attention(q, kk, v, [0], F, Hs, Ws, k, 0.37)
        want = _brute(_f64(q[0, 0]).tolist(), _f64(kk[0, 0]).tolist(), _f64(v[0, 0]).tolist(), F, Hs, Ws, k, 0.37)
        np.testing.assert_allclose(got[0, 0], want, rtol=1e-12, atol=1e-13)
    except AssertionError:
        return False
    return True


class _Mutant:
    def __init__(self, **over):
        self.__dict__.update({n: getattr(A, n) for n in dir(A) if not n.startswith("__")})
        self.__dict__.update(over)
        # rebuild the dependent functions so that they see the overrides
        src = open(A.__file__).read()
        env = {"__name__": "oracle.anchor_mutant", "__package__": "oracle"}
        exec(compile(src, A.__file__, "exec"), env)
        env.update(over)
        for name in ("nearest_anchor", "anchor_token_maps", "anchor_attention", "anchor_rows", "dense_rows"):
            if name not in over:
                fn = env[name]
                self.__dict__[name] = type(fn)(fn.__code__, env, name, fn.__defaults__, fn.__closure__)
            else:
                env[name] = over[name]


def test_the_unmodified_oracle_passes_the_mutant_harness():
    assert _run_pins(_Mutant())


@pytest.mark.parametrize(
    "name,over",
    [
        ("anchors at segment starts", dict(anchor_rows=lambda n, k: np.array([(j * n) // k for j in range(k)], dtype=np.int64))),
        ("anchors at segment ends", dict(anchor_rows=lambda n, k: np.array([((j + 1) * n) // k - 1 for j in range(k)], dtype=np.int64))),
        ("ties to the upper anchor", dict(nearest_anchor=lambda n, k: np.array(
            [max(range(k), key=lambda j: (-abs(y - int(A.anchor_rows(n, k)[j])), j)) for y in range(n)], dtype=np.int64))),
        ("no max subtraction, wrong normaliser", dict(dense_rows=lambda q, k, v, s: (np.exp(s * (q @ k.T)) / np.exp(s * (q @ k.T)).sum(axis=0, keepdims=True)) @ v)),
        ("scale dropped", dict(dense_rows=lambda q, k, v, s: A.dense_rows(q, k, v, 1.0))),
        ("keys and values swapped", dict(dense_rows=lambda q, k, v, s: A.dense_rows(q, v, k, s))),
    ],
)
def test_mutants_fail(name, over):
    assert not _run_pins(_Mutant(**over)), name
