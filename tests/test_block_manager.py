"""Host logic of the paged KV manager (no GPU): sharing, copy on write, tail cut, conservation,
and a model check against a naive copy-everything implementation on random traces."""
import numpy as np
import pytest

from paper_2605_10380_amd import binding as B
from paper_2605_10380_amd import inputs as I

Bk = 16


@pytest.fixture
def pool():
    cfg = B.make_config(I.SHAPES["tiny"], 4096, 64)
    p = B.ax_pool_create(cfg, 0, B.ax_pool_block_bytes(cfg) * 64)
    yield p
    # every test frees its sequences: the pool must be destroyable and full again
    free, total, live = B.ax_pool_stats(p)
    assert (free, live) == (total, 0)
    B.ax_pool_destroy(p)


def test_block_bytes_match_the_papers_7b_figure():
    cfg = B.make_config(I.SHAPES["8b"], 16384, 64)
    assert B.ax_pool_block_bytes(cfg) == 16 * 131072       # 128 KiB per token (paper Sec. 5.5)


def test_alloc_grow_truncate_free(pool):
    kv = B.ax_kv_alloc(pool)
    assert B.ax_kv_len(kv) == 0 and len(B.ax_kv_blocks(kv)) == 0
    assert B.ax_kv_reserve_host(kv, 40) == (-1, -1)
    assert B.ax_kv_len(kv) == 40 and list(B.ax_kv_blocks(kv)) == [0, 1, 2]   # consecutive blocks
    B.ax_kv_truncate(kv, 33)
    assert len(B.ax_kv_blocks(kv)) == 3
    B.ax_kv_truncate(kv, 32)                                 # block 2 is wholly beyond the cut
    assert list(B.ax_kv_blocks(kv)) == [0, 1] and B.ax_pool_stats(pool)[0] == 62
    B.ax_kv_truncate(kv, 0)
    assert len(B.ax_kv_blocks(kv)) == 0
    with pytest.raises(B.AxError):
        B.ax_kv_truncate(kv, 1)                              # cannot grow by truncate
    B.ax_kv_free(kv)


def test_fork_shares_blocks_and_append_copies_shared_tail(pool):
    a = B.ax_kv_alloc(pool)
    B.ax_kv_reserve_host(a, 40)
    f = B.ax_kv_fork(a, 20)                                  # shares blocks 0 and 1
    assert list(B.ax_kv_blocks(f)) == [0, 1]
    assert [B.ax_pool_refcount(pool, b) for b in (0, 1, 2)] == [2, 2, 1]
    free_before = B.ax_pool_stats(pool)[0]
    src, dst = B.ax_kv_reserve_host(f, 1)                    # slot 4 of block 1 belongs to `a` too
    assert src == 1 and dst not in (0, 1, 2)
    assert list(B.ax_kv_blocks(f)) == [0, dst] and list(B.ax_kv_blocks(a)) == [0, 1, 2]
    assert [B.ax_pool_refcount(pool, b) for b in (0, 1, dst)] == [2, 1, 1]
    assert B.ax_pool_stats(pool)[0] == free_before - 1
    assert B.ax_kv_reserve_host(f, 1) == (-1, -1)            # now private: no second copy
    # a fork cut at a block boundary never copies
    g = B.ax_kv_fork(a, 32)
    assert B.ax_kv_reserve_host(g, 5) == (-1, -1)
    assert list(B.ax_kv_blocks(g))[:2] == [0, 1]
    # the source itself copies when ITS partly filled tail is shared
    h = B.ax_kv_fork(a)                                      # all 40 tokens, block 2 shared
    s2, d2 = B.ax_kv_reserve_host(a, 1)
    assert s2 == 2 and list(B.ax_kv_blocks(h)) == [0, 1, 2] and B.ax_kv_blocks(a)[2] == d2
    with pytest.raises(B.AxError):
        B.ax_kv_fork(a, 1000)
    for k in (a, f, g, h):
        B.ax_kv_free(k)


def test_oom_leaves_everything_unchanged(pool):
    a = B.ax_kv_alloc(pool)
    B.ax_kv_reserve_host(a, 64 * Bk - 8)                     # all 64 blocks, last one half full
    f = B.ax_kv_fork(a)
    before = (B.ax_kv_len(f), list(B.ax_kv_blocks(f)), B.ax_pool_stats(pool))
    with pytest.raises(B.AxError) as e:
        B.ax_kv_reserve_host(f, 1)                           # would need a copy, none free
    assert e.value.status == B.AX_ERR_OOM
    assert before == (B.ax_kv_len(f), list(B.ax_kv_blocks(f)), B.ax_pool_stats(pool))
    B.ax_kv_free(a)
    assert B.ax_kv_reserve_host(f, 1) == (-1, -1)            # sole owner now: in place
    B.ax_kv_free(f)


def test_bad_handles_are_rejected(pool):
    kv = B.ax_kv_alloc(pool)
    B.ax_kv_free(kv)
    with pytest.raises(B.AxError):
        B.ax_kv_free(kv)                                     # double free
    assert B.ax_kv_len(kv) == -1
    with pytest.raises(B.AxError):
        B.ax_kv_alloc(0)
    live = B.ax_kv_alloc(pool)
    with pytest.raises(B.AxError) as e:
        B.ax_pool_destroy(pool)
    assert e.value.status == B.AX_ERR_STATE
    B.ax_kv_free(live)


class NaiveSeq:
    """Copy-everything model: a sequence is a list of (owner tag, position) cells."""
    def __init__(self, cells=None):
        self.cells = list(cells or [])


@pytest.mark.parametrize("seed", range(5))
def test_random_traces_against_naive_model(seed):
    """Refcounts always equal the number of sequences holding each block, the free count is
    conserved, and the cells a sequence can read are exactly those of the naive model: a block
    is shared only where the content (who wrote which position) is identical."""
    rng = np.random.default_rng(seed)
    cfg = B.make_config(I.SHAPES["tiny"], 1 << 20, 64)
    n_blocks = 96
    pool = B.ax_pool_create(cfg, 0, B.ax_pool_block_bytes(cfg) * n_blocks)
    content = {}                    # (block, slot) -> tag written there
    seqs = []                       # (handle, NaiveSeq)
    tag = 0
    for step in range(400):
        op = rng.choice(["alloc", "append", "fork", "trunc", "free"], p=[0.1, 0.4, 0.2, 0.2, 0.1])
        if op == "alloc" or not seqs:
            seqs.append((B.ax_kv_alloc(pool), NaiveSeq()))
        elif op == "append":
            h, m = seqs[rng.integers(len(seqs))]
            n = int(rng.integers(1, 40))
            before = (B.ax_kv_len(h), list(B.ax_kv_blocks(h)), B.ax_pool_stats(pool)[0])
            try:
                src, dst = B.ax_kv_reserve_host(h, n)
            except B.AxError as e:
                assert e.status == B.AX_ERR_OOM
                assert before == (B.ax_kv_len(h), list(B.ax_kv_blocks(h)), B.ax_pool_stats(pool)[0])
                continue
            if src >= 0:
                for s in range(Bk):
                    if (src, s) in content:
                        content[(dst, s)] = content[(src, s)]
            blocks = B.ax_kv_blocks(h)
            for pos in range(len(m.cells), len(m.cells) + n):
                tag += 1
                m.cells.append(tag)
                blk = int(blocks[pos // Bk])
                assert B.ax_pool_refcount(pool, blk) == 1      # never write into a shared block
                content[(blk, pos % Bk)] = tag
        elif op == "fork":
            h, m = seqs[rng.integers(len(seqs))]
            n = int(rng.integers(0, len(m.cells) + 1))
            seqs.append((B.ax_kv_fork(h, n), NaiveSeq(m.cells[:n])))
        elif op == "trunc":
            h, m = seqs[rng.integers(len(seqs))]
            n = int(rng.integers(0, len(m.cells) + 1))
            B.ax_kv_truncate(h, n)
            m.cells = m.cells[:n]
        else:
            i = int(rng.integers(len(seqs)))
            B.ax_kv_free(seqs[i][0])
            seqs.pop(i)
        # invariants
        held = np.zeros(n_blocks, dtype=int)
        for h, m in seqs:
            blocks = B.ax_kv_blocks(h)
            assert B.ax_kv_len(h) == len(m.cells) and len(blocks) == -(-len(m.cells) // Bk)
            for b in blocks:
                held[b] += 1
            for pos, t in enumerate(m.cells):
                assert content[(int(blocks[pos // Bk]), pos % Bk)] == t
        assert all(B.ax_pool_refcount(pool, b) == held[b] for b in range(n_blocks))
        free, total, live = B.ax_pool_stats(pool)
        assert free == n_blocks - np.count_nonzero(held) and live == len(seqs)
    for h, _ in seqs:
        B.ax_kv_free(h)
    assert B.ax_pool_stats(pool)[0] == n_blocks
    B.ax_pool_destroy(pool)
