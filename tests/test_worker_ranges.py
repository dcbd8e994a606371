"""The partition of the flat tile space among the persistent workers, computed on the host by the
code the kernels run (kv_worker_range / kv_worker_of_tile): exact against integer arithmetic, a
partition, and inverted correctly, also for tile counts far beyond what a GPU test can hold."""
import random

import pytest

import paper_2504_06319_amd as kv


def weight(w, skew):
    return 1024 * w + skew * (w & 1)


def exact_start(w, tiles, nw, skew):
    return tiles * weight(w, skew) // weight(nw, skew)


def cases():
    rng = random.Random(20250408)
    out = [(1, 1, 0), (1, 512, 20), (511, 512, 20), (512, 512, 20), (16 * 512 - 1, 512, 20), (16 * 512, 512, 20), (64 * 512, 512, 20),
           (126416, 512, 20), (126416, 1536, 20), (63344, 1536, 20), (2**31 - 1, 4096, 256), (2**40, 4095, 255),
           (2**40, 4096, 0), (2**36 + 12345, 1, 20), (100003, 7, 256)]
    for _ in range(300):
        nw = rng.choice([1, 2, 3, 255, 256, 511, 512, 1024, 1536, 4095, 4096, rng.randint(1, 4096)])
        tiles = rng.choice([rng.randint(1, 4 * nw), rng.randint(nw, 10**6), rng.randint(10**6, 2**40)])
        out.append((tiles, nw, rng.choice([0, 1, 20, 100, 256])))
    return out


@pytest.mark.parametrize("tiles,workers,skew", cases())
def test_ranges_partition_the_tile_space_exactly(tiles, workers, skew):
    nw = min(tiles, workers)
    eff = skew if tiles >= 16 * nw else 0          # short ranges are not skewed
    rng = random.Random(tiles ^ workers)
    sample = sorted({0, 1, nw // 2, nw - 2, nw - 1} | {rng.randrange(nw) for _ in range(40)})
    prev_end = None
    for w in [x for x in sample if 0 <= x < nw]:
        first, end = kv.kv_worker_range(tiles, workers, skew, w)
        assert first == exact_start(w, tiles, nw, eff) and end == exact_start(w + 1, tiles, nw, eff)
        assert first < end                          # every active worker has at least one tile
        if w == 0:
            assert first == 0
        if w == nw - 1:
            assert end == tiles
        # inverse, at both ends of the range and just outside
        assert kv.kv_worker_of_tile(tiles, workers, skew, first) == w
        assert kv.kv_worker_of_tile(tiles, workers, skew, end - 1) == w
        if first > 0:
            assert kv.kv_worker_of_tile(tiles, workers, skew, first - 1) == w - 1
        if end < tiles:
            assert kv.kv_worker_of_tile(tiles, workers, skew, end) == w + 1
        if prev_end is not None and prev_end[0] == w - 1:
            assert prev_end[1] == first             # contiguous
        prev_end = (w, end)


def test_small_spaces_are_covered_tile_by_tile():
    for tiles, workers, skew in [(1, 4, 20), (5, 8, 20), (97, 8, 256), (1000, 7, 20), (64 * 6, 6, 256), (700, 6, 256)]:
        nw = min(tiles, workers)
        owner = [kv.kv_worker_of_tile(tiles, workers, skew, t) for t in range(tiles)]
        assert owner == sorted(owner) and owner[0] == 0 and owner[-1] == nw - 1
        for w in range(nw):
            first, end = kv.kv_worker_range(tiles, workers, skew, w)
            assert owner[first:end] == [w] * (end - first) and owner.count(w) == end - first


def test_skew_moves_shares_between_even_and_odd_workers():
    tiles, workers = 126416, 512
    size = lambda w, s: (lambda r: r[1] - r[0])(kv.kv_worker_range(tiles, workers, s, w))
    assert {size(w, 0) for w in range(workers)} <= {246, 247}
    even = sum(size(w, 20) for w in range(0, workers, 2)) / 256
    odd = sum(size(w, 20) for w in range(1, workers, 2)) / 256
    assert abs(even / odd - (1024 + 20) / (1024 - 20)) < 2e-3


def test_invalid_arguments():
    with pytest.raises(kv.KVError):
        kv.kv_worker_range(0, 512, 20, 0)
    with pytest.raises(kv.KVError):
        kv.kv_worker_range(100, 512, 20, 100)       # only min(tiles, workers) workers are active
    with pytest.raises(kv.KVError):
        kv.kv_worker_range(100, 512, 257, 0)
    assert kv.kv_worker_of_tile(100, 512, 20, 100) == -1
    assert kv.kv_worker_of_tile(100, 0, 20, 5) == -1
