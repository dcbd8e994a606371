"""Closed forms of the paper's working-set analysis (Section 3.3).

TEST INFRASTRUCTURE ONLY.
"""


def block_bytes(bytes_per_element: int, head_dim: int, tokens_per_block: int) -> int:
    """Eq. 1: footprint of one K (or V) block of one head."""
    return bytes_per_element * head_dim * tokens_per_block


def iteration_working_set_bytes(m_block: int, n_thread: int, heads: int, batch: int,
                                lanes_per_wave: int = 32) -> int:
    """Eq. 2: bytes of blocks touched per loop iteration by the whole grid.

    n_thread / lanes_per_wave is the number of waves of a thread block, each of which
    owns one block per iteration; the grid has heads x batch thread blocks.  Sequence
    length does not appear.
    """
    assert n_thread % lanes_per_wave == 0
    return m_block * (n_thread // lanes_per_wave) * heads * batch


def max_resident_batches(cache_bytes: int, per_batch_working_set: int) -> int:
    """Largest batch whose per-iteration working set still fits the cache (Section 3.3)."""
    return cache_bytes // per_batch_working_set
