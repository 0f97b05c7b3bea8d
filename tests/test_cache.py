"""Activation cache (Section 4.3 of the paper, Figure 6: a table in GPU memory
keyed by sample id, holding the recent mini-batches' activations): pins of the
CPU oracle against what the description fixes, then the library's kernels
against the oracle through the C-ABI (bit-exact: it is index and copy work)."""
import numpy as np
import pytest

from oracle.cache_oracle import CacheOracle


def rows_for(ids, D, salt=0):
    """A row that is a known function of (id, salt), so that a served row names its origin."""
    ids = np.asarray(ids, np.int64)
    return (ids[:, None] * 1000 + salt * 100 + np.arange(D)[None, :]).astype(np.float32)


# ----------------------------------------------------------------------------- oracle pins

def test_oracle_keeps_the_recent_five_minibatches():
    o, D = CacheOracle(5), 3
    for t in range(6):                                  # six mini-batches of disjoint ids
        ids = np.arange(4) + 10 * t
        o.put(ids, rows_for(ids, D))
    out = np.full((4, D), -1.0, np.float32)
    assert o.get(np.arange(4), out).tolist() == [0, 0, 0, 0]     # the first one is gone
    assert (out == -1.0).all()                                    # and its rows untouched
    for t in range(1, 6):
        ids = np.arange(4) + 10 * t
        out = np.zeros((4, D), np.float32)
        assert o.get(ids, out).tolist() == [1, 1, 1, 1]
        assert np.array_equal(out, rows_for(ids, D))


def test_oracle_newer_put_wins_and_outlives_the_older_minibatch():
    o, D = CacheOracle(2), 2
    o.put([7, 8], rows_for([7, 8], D, salt=1))
    o.put([7, 9], rows_for([7, 9], D, salt=2))
    out = np.zeros((3, D), np.float32)
    assert o.get([7, 8, 9], out).tolist() == [1, 1, 1]
    assert np.array_equal(out[0], rows_for([7], D, salt=2)[0])    # served from the newer mini-batch
    o.put([1, 2], rows_for([1, 2], D, salt=3))                    # drops the first mini-batch
    out = np.zeros((3, D), np.float32)
    assert o.get([7, 8, 9], out).tolist() == [1, 0, 1]
    assert np.array_equal(out[0], rows_for([7], D, salt=2)[0])


def test_oracle_repeated_and_negative_ids():
    o, D = CacheOracle(5), 2
    rows = np.array([[1, 1], [2, 2], [3, 3], [4, 4]], np.float32)
    o.put([5, -1, 5, -7], rows)
    out = np.zeros((3, D), np.float32)
    assert o.get([5, -1, -7], out).tolist() == [1, 0, 0]
    assert out[0].tolist() == [3, 3]                              # the last row of the repeated id


def replay_reference(history, window, query, D):
    """What the description fixes, written the other way round: replay the last
    `window` mini-batches in order into one plain table, later rows overwrite."""
    table = {}
    for ids, rows in history[-window:]:
        for i, k in enumerate(ids):
            if k >= 0:
                table[int(k)] = rows[i]
    hit = np.array([1 if int(k) in table else 0 for k in query], np.uint8)
    return hit, table


@pytest.mark.parametrize("window,batch,universe", [(1, 3, 5), (5, 8, 30), (3, 16, 20), (5, 4, 1000)])
def test_oracle_against_replay(window, batch, universe):
    rng = np.random.default_rng(window * 100 + batch)
    o, D, history = CacheOracle(window), 4, []
    for t in range(25):
        n = int(rng.integers(0, batch + 1))
        ids = rng.integers(-2, universe, size=n)
        rows = rng.standard_normal((n, D)).astype(np.float32)
        o.put(ids, rows)
        history.append((ids, rows))
        query = rng.integers(-2, universe, size=12)
        out = np.full((12, D), 9.0, np.float32)
        hit = o.get(query, out)
        want_hit, table = replay_reference(history, window, query, D)
        assert np.array_equal(hit, want_hit)
        for i, k in enumerate(query):
            assert np.array_equal(out[i], table[int(k)] if hit[i] else np.full(D, 9.0, np.float32))
