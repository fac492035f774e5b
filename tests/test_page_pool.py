"""Host-side page pool: a window layer's cache stays bounded by its window (CPU only).

The bound is the paper's: with window attention the per-layer KV footprint is proportional to W,
not to the context length (Section 2, "Window attention for long-context inference")."""
import numpy as np
import pytest

import paper_2602_11937_amd as pz


def test_window_pages_closed_form():
    # brute force: the most pages any window [L-W, L) can touch
    for W in (1, 2, 15, 16, 17, 20, 128, 129, 8192):
        for P in (16, 32, 64):
            worst = max(((L - 1) // P) - (max(L - W, 0) // P) + 1 for L in range(1, 4 * P + W + 2))
            assert pz.pz_window_pages(W, P) == worst, (W, P)
    assert pz.pz_window_pages(0, 64) == 0 and pz.pz_window_pages(128, 64) == 3


@pytest.mark.parametrize("W,P", [(20, 16), (128, 64), (16, 16), (1, 16), (100, 32)])
def test_window_layer_never_holds_more_than_its_window(W, P):
    n_seq, steps = 5, 700
    per_seq = pz.pz_window_pages(W, P)
    pool = pz.PagePool(n_seq * per_seq, P, n_seq, (steps + P) // P + 1, window=W)
    mirror = np.full(pool.shape, -1, dtype=np.int32)                  # what a device table would hold
    rng = np.random.default_rng(W * P)
    lens = [0] * n_seq
    for _ in range(steps):
        b = int(rng.integers(n_seq))
        slot = pool.append(b)
        lens[b] += 1
        idx, val = pool.drain_updates()
        mirror.reshape(-1)[idx] = val
        table = pool.block_table()
        assert np.array_equal(mirror, table) and pool.seq_len(b) == lens[b]
        pos = lens[b] - 1
        assert slot == int(table[b, pos // P]) * P + pos % P
        live = []
        for s in range(n_seq):                                       # every attended page is valid, no page shared
            if lens[s] == 0:
                continue
            lo = max(lens[s] - W, 0)
            pages = table[s, lo // P:(lens[s] - 1) // P + 1]
            assert np.all(pages >= 0) and len(pages) <= per_seq
            held = table[s][table[s] >= 0]
            assert len(held) <= per_seq
            live += held.tolist()
        assert len(live) == len(set(live)) and pool.free_pages() == n_seq * per_seq - len(live)
    pool.release(2)
    assert pool.seq_len(2) == 0 and np.all(pool.block_table()[2] == -1)
    pool.close()


def test_full_attention_pool_grows_and_runs_out():
    pool = pz.PagePool(3, 16, 2, 8, window=0)
    for _ in range(33):
        assert pool.append(0) >= 0                                   # 33 positions: 3 pages
    assert pool.free_pages() == 0
    assert pool.append(1, check=False) == -4                         # PZ_ERR_WORKSPACE: no page left
    for _ in range(15):
        assert pool.append(0) >= 0                                   # the open page still has room
    assert pool.append(0, check=False) == -4
    pool.release(0)
    assert pool.free_pages() == 3 and pool.append(1) >= 0
    assert pool.append(5, check=False) == -2                         # bad sequence id
    pool.close()
    tiny = pz.PagePool(8, 16, 1, 2, window=0)
    for _ in range(32):
        tiny.append(0)
    assert tiny.append(0, check=False) == -2                         # block-table row is full
    tiny.close()
    with pytest.raises(pz.PzError):
        pz.PagePool(0, 16, 1, 1)


def test_a_refused_append_changes_nothing_and_a_window_step_can_reuse_its_own_page():
    """Errors are found before the pool changes (so a caller may retry after releasing something), and the
    one case where an empty free list is not an error: the step itself hands back the page it then opens."""
    pool = pz.PagePool(2, 16, 2, 64, window=17)                      # 17 positions touch at most 2 pages
    for _ in range(32):
        assert pool.append(0) >= 0                                   # positions 0..31: pages 0 and 1, nothing free
    assert pool.free_pages() == 0
    table, pending = pool.block_table().copy(), pool.drain_updates()
    assert pool.append(1, check=False) == -4                         # another sequence: refused
    assert np.array_equal(pool.block_table(), table) and pool.seq_len(1) == 0 and len(pool.drain_updates()[0]) == 0
    slot = pool.append(0)                                            # position 32 opens a page: page 0 of the
    assert slot // 16 == table[0, 0]                                 # sequence left the window and comes back
    idx, val = pool.drain_updates()
    assert list(idx) == [0, 2] and list(val) == [-1, int(table[0, 0])]
    assert pool.seq_len(0) == 33 and pool.free_pages() == 0
    pool.close()
    assert pz.lib().pz_page_pool_create(4, 16, 70000, 70000, 0) is None     # table indices would pass 32 bits
