"""Host-only tests of the unified page pool: page geometry, growth of FA caches, bounded SWA caches,
fixed recurrent pages, exhaustion, reuse, and the kernel-facing tables."""
import numpy as np
import pytest

from paper_2604_19877_amd import binding as sa

SHAPES = sa.sa_shapes(32, 32, 128, 128, 32, 8, 128, 16)


@pytest.fixture
def pool():
    p = sa.sa_pool_create(40, SHAPES, 4)
    yield p
    sa.sa_pool_destroy(p)


def all_pages(pool, seqs, max_pages=192):
    """Unified pages referenced by the tables of every layer (recurrent slots and KV pages)."""
    stride = sa.sa_pool_kv_id_stride(pool)
    used = []
    for layer in range(4):
        table, slot = sa.sa_pool_layer_tables(pool, seqs, layer, max_pages)
        used += [int(s) for s in slot if s >= 0]
        for row in table:
            used += sorted({int(e) // stride for e in row if e >= 0})
    return used


def test_geometry_follows_the_15b_shapes(pool):
    # one page = one 32 x 128 x 128 fp32 state = 2 MiB = K and V (8 heads, bf16) of 512 tokens
    assert sa.sa_pool_page_bytes(pool) == 32 * 128 * 128 * 4 == 2 << 20
    assert sa.sa_pool_tokens_per_page(pool) == 512
    assert sa.sa_pool_kv_id_stride(pool) == 64
    # the kernels' page bound: the last id whose V block (half a unified page behind its K block) is still in the arena, + 1
    assert sa.sa_pool_kernel_pages(pool) == 40 * 64 - 32
    last = sa.sa_pool_kernel_pages(pool) - 1
    block = 8 * 16 * 128 * 2
    assert (2 << 20) // 2 + (last + 1) * block == 40 * (2 << 20)
    assert sa.sa_pool_free_pages(pool) == 40


def test_growth_window_and_release(pool):
    s = sa.sa_pool_seq_create(pool, "FSKG")
    assert sa.sa_pool_seq_pages(pool, s) == 2 and sa.sa_pool_free_pages(pool) == 38     # K and G state pages
    sa.sa_pool_seq_reserve(pool, s, 1, 1024)
    assert sa.sa_pool_seq_pages(pool, s) == 4                                            # first page of F and of S
    sa.sa_pool_seq_reserve(pool, s, 512, 1024)
    assert sa.sa_pool_seq_pages(pool, s) == 4
    sa.sa_pool_seq_reserve(pool, s, 513, 1024)
    assert sa.sa_pool_seq_pages(pool, s) == 6
    sa.sa_pool_seq_reserve(pool, s, 4000, 1024)
    # F holds ceil(4000/512) = 8 pages; S holds the pages touching tokens [2976, 4000): blocks 5..7 = 3 pages
    assert sa.sa_pool_seq_pages(pool, s) == 2 + 8 + 3
    table, slot = sa.sa_pool_layer_tables(pool, [s], 1, 256)
    assert (table[0, :5 * 32] == -1).all() and (table[0, 5 * 32:8 * 32] >= 0).all() and (table[0, 8 * 32:] == -1).all()
    assert slot[0] == -1
    table_f, _ = sa.sa_pool_layer_tables(pool, [s], 0, 256)
    assert (table_f[0, :256] >= 0).all()
    # kernel page ids: 32 consecutive ids per unified page, unified pages 64 ids apart
    ids = table_f[0, :64]
    assert (np.diff(ids[:32]) == 1).all() and ids[0] % 64 == 0 and ids[32] % 64 == 0 and ids[32] != ids[0] + 32
    _, slot_k = sa.sa_pool_layer_tables(pool, [s], 2, 0)
    _, slot_g = sa.sa_pool_layer_tables(pool, [s], 3, 0)
    assert slot_k[0] >= 0 and slot_g[0] >= 0 and slot_k[0] != slot_g[0]
    used = all_pages(pool, [s], 256)
    assert len(used) == len(set(used)) == 13 and sa.sa_pool_free_pages(pool) == 40 - 13
    sa.sa_pool_seq_free(pool, s)
    assert sa.sa_pool_free_pages(pool) == 40 and sa.sa_pool_seq_pages(pool, s) == -1


def test_pages_are_never_shared_between_sequences(pool):
    seqs = [sa.sa_pool_seq_create(pool, p) for p in ("FFSS", "KGKG", "SFGK")]
    for s, n in zip(seqs, (1500, 9000, 700)):
        sa.sa_pool_seq_reserve(pool, s, n, 600, slack=3)
    used = all_pages(pool, seqs)
    assert len(used) == len(set(used)) == 40 - sa.sa_pool_free_pages(pool)
    assert sum(sa.sa_pool_seq_pages(pool, s) for s in seqs) == len(used)
    sa.sa_pool_seq_free(pool, seqs[1])
    s4 = sa.sa_pool_seq_create(pool, "FFFF")
    assert s4 == seqs[1]                               # the id is reused
    sa.sa_pool_seq_reserve(pool, s4, 1024, 600)
    used = all_pages(pool, [seqs[0], s4, seqs[2]])
    assert len(used) == len(set(used))


def test_exhaustion_changes_nothing(pool):
    s = sa.sa_pool_seq_create(pool, "FFFF")
    sa.sa_pool_seq_reserve(pool, s, 512 * 9, 4096)     # 36 pages
    before = (sa.sa_pool_free_pages(pool), sa.sa_pool_seq_pages(pool, s))
    assert before == (4, 36)
    with pytest.raises(sa.SaError) as e:
        sa.sa_pool_seq_reserve(pool, s, 512 * 11, 4096)
    assert e.value.status == sa.SA_ENOMEM
    assert (sa.sa_pool_free_pages(pool), sa.sa_pool_seq_pages(pool, s)) == before


def test_exhaustion_on_create(pool):
    s = sa.sa_pool_seq_create(pool, "FFFF")
    sa.sa_pool_seq_reserve(pool, s, 512 * 9, 4096)
    a = sa.sa_pool_seq_create(pool, "KGKG")            # takes the last 4 pages
    assert sa.sa_pool_free_pages(pool) == 0
    with pytest.raises(sa.SaError) as e:
        sa.sa_pool_seq_create(pool, "FFFK")
    assert e.value.status == sa.SA_ENOMEM
    sa.sa_pool_seq_create(pool, "FFFF")                # needs nothing yet
    sa.sa_pool_seq_free(pool, a)
    assert sa.sa_pool_free_pages(pool) == 4


def test_a_sliding_window_sequence_runs_forever_in_bounded_space(pool):
    s = sa.sa_pool_seq_create(pool, "SSSS")
    peak = 0
    for n in range(1, 60000, 257):
        sa.sa_pool_seq_reserve(pool, s, n, 4096, slack=3)
        peak = max(peak, sa.sa_pool_seq_pages(pool, s))
    assert peak <= 4 * (4096 // 512 + 2) <= 40
    table, _ = sa.sa_pool_layer_tables(pool, [s], 0, 59904 // 16 + 8)
    n = 59881
    live = np.flatnonzero(table[0] >= 0)
    assert live.min() * 16 <= n - 4096 - 3 and live.max() * 16 + 16 >= n


def test_a_length_jump_past_the_window_on_a_nearly_full_pool():
    # An F layer ahead of an S layer, 7 pages, window 1024: the second reserve needs 3 more pages for F while only 2 are
    # free; the third comes from the S layer, whose first two blocks fall behind the window.  Every S layer has to give
    # before any layer takes, or the F layer empties the free list and pages end up mapped twice.
    p = sa.sa_pool_create(7, SHAPES, 2)
    try:
        s = sa.sa_pool_seq_create(p, "FS")
        sa.sa_pool_seq_reserve(p, s, 1535, 1024)                   # blocks 0..2 on both layers: 6 pages, 1 free
        assert (sa.sa_pool_free_pages(p), sa.sa_pool_seq_pages(p, s)) == (1, 6)
        sa.sa_pool_seq_reserve(p, s, 2560, 1024)                   # F: blocks 0..4; S: tokens [1536, 2560) = blocks 3..4
        assert (sa.sa_pool_free_pages(p), sa.sa_pool_seq_pages(p, s)) == (0, 7)
        stride = sa.sa_pool_kv_id_stride(p)
        used = []
        for layer in range(2):
            table, _ = sa.sa_pool_layer_tables(p, [s], layer, 5 * 32)
            used += sorted({int(e) // stride for e in table[0] if e >= 0})
        assert sorted(used) == list(range(7))                      # every page exactly once
        table_s, _ = sa.sa_pool_layer_tables(p, [s], 1, 5 * 32)
        assert (table_s[0, :3 * 32] == -1).all() and (table_s[0, 3 * 32:] >= 0).all()
        # one page too many: refused, nothing changes
        with pytest.raises(sa.SaError) as e:
            sa.sa_pool_seq_reserve(p, s, 3073, 1024)
        assert e.value.status == sa.SA_ENOMEM
        assert (sa.sa_pool_free_pages(p), sa.sa_pool_seq_pages(p, s)) == (0, 7)
        sa.sa_pool_seq_free(p, s)
        assert sa.sa_pool_free_pages(p) == 7
    finally:
        sa.sa_pool_destroy(p)


def test_random_reserves_keep_the_books_balanced():
    rng = np.random.default_rng(77)
    for trial in range(20):
        n_pages, L = int(rng.integers(6, 30)), int(rng.integers(1, 5))
        p = sa.sa_pool_create(n_pages, SHAPES, L)
        try:
            seqs = {}
            for _ in range(60):
                if seqs and rng.random() < 0.15:
                    s = list(seqs)[int(rng.integers(len(seqs)))]
                    sa.sa_pool_seq_free(p, s)
                    del seqs[s]
                elif len(seqs) < 3 and rng.random() < 0.3:
                    try:
                        seqs[sa.sa_pool_seq_create(p, "".join(rng.choice(list("FSKG"), L)))] = 0
                    except sa.SaError as e:
                        assert e.status == sa.SA_ENOMEM
                elif seqs:
                    s = list(seqs)[int(rng.integers(len(seqs)))]
                    n = seqs[s] + int(rng.integers(1, 3000))
                    before = (sa.sa_pool_free_pages(p), sa.sa_pool_seq_pages(p, s))
                    try:
                        sa.sa_pool_seq_reserve(p, s, n, int(rng.integers(1, 2000)), int(rng.integers(0, 4)))
                        seqs[s] = n
                    except sa.SaError as e:
                        assert e.status == sa.SA_ENOMEM
                        assert (sa.sa_pool_free_pages(p), sa.sa_pool_seq_pages(p, s)) == before
                held = sum(sa.sa_pool_seq_pages(p, s) for s in seqs)
                assert held + sa.sa_pool_free_pages(p) == n_pages
                stride = sa.sa_pool_kv_id_stride(p)
                used = []
                for layer in range(L):
                    table, slot = sa.sa_pool_layer_tables(p, list(seqs), layer, max(seqs.values(), default=0) // 16 + 32)
                    used += [int(x) for x in slot if x >= 0]
                    for row in table:
                        used += sorted({int(e) // stride for e in row if e >= 0})
                assert len(used) == len(set(used)) == held
        finally:
            sa.sa_pool_destroy(p)


def test_argument_errors(pool):
    for bad in ("FSK", "FSKX"):
        with pytest.raises(sa.SaError) as e:
            sa.sa_pool_seq_create(pool, bad)
        assert e.value.status == sa.SA_EINVAL
    with pytest.raises(sa.SaError):
        sa.sa_pool_seq_reserve(pool, 7, 10, 10)
    with pytest.raises(sa.SaError):
        sa.sa_pool_seq_free(pool, 0)
    with pytest.raises(sa.SaError) as e:
        sa.sa_pool_create(4, sa.sa_shapes(3, 3, 10, 10, 32, 8, 128, 16), 2)      # 1200-byte state: not a whole K+V page
    assert e.value.status == sa.SA_EUNSUPPORTED
