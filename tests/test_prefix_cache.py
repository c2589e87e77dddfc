"""Block-level prefix cache: matching, sharing, reference counts, eviction order."""
import numpy as np
import pytest

from paper_2601_11546_amd.prefix_cache import BlockPrefixCache


def _toks(template, suffix_seed, n_suffix):
    rng = np.random.default_rng(suffix_seed)
    return np.concatenate([template, rng.integers(0, 1000, n_suffix).astype(np.int32)])


def test_requests_behind_one_template_share_its_blocks():
    c = BlockPrefixCache(64, 16)
    template = np.arange(64, dtype=np.int32)                    # 4 full blocks
    a = _toks(template, 1, 20)
    assert c.match(a) == 0
    pa, cached, ready = c.acquire(a, 5)
    assert cached == 0 and ready == 0 and len(pa) == (84 + 5 + 15) // 16
    b = _toks(template, 2, 30)
    assert c.match(b) == 64                                     # the template, registered when a was admitted
    pb, cached, ready = c.acquire(b, 5)
    assert cached == 64 and ready == 0 and pb[:4] == pa[:4] and not set(pb[4:]) & set(pa)     # same batch: not ready yet
    c.mark_ready(pa)
    pc, cached, ready = c.acquire(_toks(template, 3, 10), 5)
    assert cached == 64 and ready == 64 and pc[:4] == pa[:4]
    c.check()
    assert c.hits == 128 and c.misses == 84 + 30 + 10


def test_a_block_matches_only_behind_the_same_prefix():
    c = BlockPrefixCache(64, 16)
    x = np.arange(48, dtype=np.int32)
    c.acquire(x, 0)
    y = np.concatenate([np.full(16, 7, np.int32), x[16:]])       # same second and third block, other first block
    assert c.match(y) == 0
    z = np.concatenate([x[:32], np.full(16, 9, np.int32), x[:16]])
    assert c.match(z) == 32


def test_the_last_token_is_always_computed():
    c = BlockPrefixCache(64, 16)
    x = np.arange(64, dtype=np.int32)
    c.acquire(x, 0)
    assert c.match(x) == 48                                      # all four blocks are cached; three are used
    assert c.match(np.concatenate([x, [5]])) == 64


def test_release_keeps_keyed_blocks_until_the_pool_needs_them_lru_first():
    c = BlockPrefixCache(8, 16)
    a, b = np.arange(32, dtype=np.int32), np.arange(100, 132, dtype=np.int32)
    pa, _, _ = c.acquire(np.concatenate([a, [1]]), 0)            # 2 keyed + 1 private page
    pb, _, _ = c.acquire(np.concatenate([b, [1]]), 0)
    c.release(pa)
    c.release(pb)
    c.check()
    assert len(c.free) == 4 and len(c.idle) == 4                 # the private pages are free, the keyed ones cached
    assert c.match(np.concatenate([a, [2]])) == 32 and c.match(np.concatenate([b, [2]])) == 32
    pa2, cached, _ = c.acquire(np.concatenate([a, [3]]), 0)      # touching a makes b the least recently used
    assert cached == 32
    c.release(pa2)
    big, _, _ = c.acquire(np.arange(500, 500 + 16 * 6, dtype=np.int32), 0)     # needs 6 pages: 4 free + evicts b's two
    assert c.match(np.concatenate([b, [2]])) == 0 and c.match(np.concatenate([a, [2]])) == 32
    c.check()
    with pytest.raises(RuntimeError):
        c.acquire(np.arange(900, 900 + 16 * 4, dtype=np.int32), 0)               # 2 idle pages left, 4 needed
    c.check()


def test_random_admissions_and_releases_keep_the_books():
    rng = np.random.default_rng(0)
    c = BlockPrefixCache(200, 16)
    templates = [rng.integers(0, 1000, 16 * int(rng.integers(1, 6))).astype(np.int32) for _ in range(5)]
    live = []
    for step in range(400):
        if live and (rng.random() < 0.45 or c.pages_available() < 20):
            c.release(live.pop(int(rng.integers(0, len(live)))))
        else:
            t = templates[int(rng.integers(0, 5))]
            toks = _toks(t, step, int(rng.integers(1, 40)))
            before = c.match(toks)
            pages, cached, ready = c.acquire(toks, int(rng.integers(0, 20)))
            assert cached == before and ready <= cached and len(set(pages)) == len(pages)
            c.mark_ready(pages)
            live.append(pages)
        c.check()
    for pages in live:
        c.release(pages)
    c.check()
    assert all(r == 0 for r in c.refs)
