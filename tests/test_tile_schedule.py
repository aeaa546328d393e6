"""The static tile schedule of the (persistent) launch, evaluated on the host through the C ABI:
every tile is processed exactly once, a workgroup's tiles stop for good at the first -1, the
workgroups of one XCD walk a contiguous range together, and under the causal mask the serpentine
order balances the per-workgroup key-tile counts."""
import pytest


@pytest.fixture(scope="module")
def sched():
    from paper_2510_14719_amd import binding
    return binding.load_library().attn_fwd_tile_schedule


def walk(sched, total, grid):
    per_block = []
    for b in range(grid):
        tiles, r = [], 0
        while True:
            t = sched(total, grid, b, r)
            if t < 0:
                assert t == -1
                break
            tiles.append(t)
            r += 1
            assert r <= total + 1
        # nothing after the first -1
        for extra in range(r + 1, r + 4):
            assert sched(total, grid, b, extra) == -1
        per_block.append(tiles)
    return per_block


@pytest.mark.parametrize("total,grid", [(1, 1), (2, 2), (7, 7), (8, 8), (9, 9), (1024, 256), (2048, 256), (1000, 256),
                                          (257, 256), (300, 256), (4099, 256), (513, 512), (96, 96), (255, 255), (5000, 304)])
def test_every_tile_exactly_once(sched, total, grid):
    per_block = walk(sched, total, grid)
    seen = sorted(t for tiles in per_block for t in tiles)
    assert seen == list(range(total))
    # balanced in tile count: no workgroup has more than one round more than another of its XCD
    for x in range(8):
        counts = [len(per_block[b]) for b in range(grid) if b % 8 == x]
        if counts:
            assert max(counts) - min(counts) <= 1


def test_one_round_is_the_xcd_contiguous_map(sched):
    total = 1024
    tiles = [sched(total, total, b, 0) for b in range(total)]
    for x in range(8):
        mine = [tiles[b] for b in range(total) if b % 8 == x]
        assert mine == list(range(x * 128, (x + 1) * 128))       # XCD x owns one contiguous range, in order
    assert all(sched(total, total, b, 1) == -1 for b in range(total))


def test_xcd_mates_walk_adjacent_tiles(sched):
    total, grid = 2048, 256
    for r in range(8):
        for x in range(8):
            row = sorted(sched(total, grid, b, r) for b in range(grid) if b % 8 == x)
            assert row == list(range(x * 256 + r * 32, x * 256 + (r + 1) * 32))


def test_argument_errors(sched):
    assert sched(0, 1, 0, 0) == -2
    assert sched(8, 9, 0, 0) == -2
    assert sched(8, 8, 8, 0) == -2
    assert sched(8, 8, 0, -1) == -2


def test_causal_lengths_balance(sched):
    # c5-like: 64 heads x 32 query tiles of 256 rows, 64-key tiles: tile qt (long first) walks 4*(32-qt) key tiles
    nqt, heads, grid = 32, 64, 256
    total = nqt * heads
    length = lambda t: 4 * (nqt - (t % nqt))
    sums = [sum(length(t) for t in tiles) for tiles in walk(sched, total, grid)]
    assert max(sums) == min(sums)                                 # even number of rounds: exact balance
    # without the serpentine order the first workgroup of an XCD would take 8 longest tiles, the last 8 shortest
    assert max(sums) < 8 * 4 * nqt * 0.6
