"""Which KV blocks one warp uses and which it fetches ahead (paper, Algorithm 1), as sets.

TEST INFRASTRUCTURE ONLY.  Stated as properties rather than as a program: of a block range
[first, end) shared by ``warps`` warps, the warp of rank r uses the blocks whose offset from
``first`` is congruent to r modulo ``warps``, in increasing order; while it computes on the
i-th of them, the fetch of the (i + distance)-th is in flight, if the warp has that many.  The
paper's algorithm is distance 1; distance 0 is its baseline (nothing is fetched ahead).
Nothing outside the range is ever named, so no block-table entry at or past ``end`` is read.
"""


def blocks_used(first: int, end: int, warps: int, rank: int) -> list:
    """Blocks the warp of this rank computes on, in the order it reaches them."""
    return [i for i in range(first, end) if (i - first) % warps == rank]


def fetches_in_flight(first: int, end: int, warps: int, rank: int, distance: int) -> dict:
    """For every block the warp computes on: the block whose fetch overlaps that computation, or None."""
    used = blocks_used(first, end, warps, rank)
    ahead = {}
    for position, block in enumerate(used):
        target = position + distance
        ahead[block] = used[target] if 0 < distance and target < len(used) else None
    return ahead
