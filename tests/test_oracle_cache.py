"""Pins of the cache model: closed forms and the paper's worked example (CPU only)."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _load_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(x) for x in line.split()])
    return rows


def test_figure_example_cache_after_each_chunk():
    # one sink, two recent, chunk 4, 16 tokens
    rows = _load_rows("fig_chunked_prefill_cache.txt")
    cache = oracle.CacheModel(sink=1, recent=2, retrieval=False)
    for row in rows:
        chunk, want = row[0], row[1:]
        for p in range(4 * chunk, 4 * chunk + 4):
            cache.append([float(p)], [float(-p)])
        assert cache.positions() == want
        assert oracle.retained_positions(4 * chunk + 4, 1, 2, False) == want
        pos, kk, vv = cache.contents()
        assert kk[:, 0].tolist() == [float(p) for p in want]
        assert vv[:, 0].tolist() == [float(-p) for p in want]


def test_kv_size_arithmetic_fixes_one_million():
    (layers, hkv, d, nbytes, tokens, total, paper_gb), = _load_rows("kv_size_llama3_8b_1m.txt")
    assert layers * hkv * d * 2 * nbytes * tokens == total
    assert round(total / 1e9) == paper_gb
    assert tokens == 2 ** 20


@pytest.mark.parametrize("sink,recent", [(0, 1), (1, 2), (4, 8), (16, 64)])
def test_mechanism_matches_closed_form(sink, recent):
    for retrieval in (False, True):
        cache = oracle.CacheModel(sink, recent, retrieval)
        for n in range(1, 3 * (sink + recent) + 5):
            cache.append([n - 1.0], [1.0 - n])
            want = oracle.retained_positions(n, sink, recent, retrieval)
            assert cache.positions() == want
            if retrieval:
                assert want == list(range(n))
            else:
                assert len(want) == min(n, sink + recent)          # constant memory
                last = list(range(max(0, n - recent), n))
                sinks = list(range(min(sink, n)))
                assert want == sorted(set(sinks) | set(last))


def test_retained_set_is_what_the_newest_query_sees():
    for n in (1, 3, 10, 50):
        for sink, recent in ((1, 2), (3, 4), (0, 5)):
            vis = oracle.visible_mask(n - 1, sink, recent, False)
            assert np.flatnonzero(vis).tolist() == oracle.retained_positions(n, sink, recent, False)
