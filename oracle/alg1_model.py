"""Index model of the paper's Algorithm 1 (prefetching K blocks), one warp's view.

TEST INFRASTRUCTURE ONLY.  The algorithm walks block indices of a range [s, e) with a
stride equal to the number of warps w; before computing on the current block it issues
a prefetch of the block the same warp will reach on its next iteration, but only when
that index is still inside the range.  The printed algorithm starts at s; here the warp
with rank r starts at s + r so that the w warps of a thread block cover the range
between them (reading noted in the design document).
"""


def alg1_trace(s: int, e: int, w: int, rank: int = 0, distance: int = 1):
    """Return (lookups, loads, prefetches) in program order for one warp.

    ``distance`` generalises "next iteration" to "k iterations ahead" (the paper is
    distance 1); distance 0 issues no prefetch at all.
    """
    lookups, loads, prefetches = [], [], []
    block_idx = s + rank
    while block_idx < e:
        lookups.append(block_idx)          # bt[block_idx] -> k_ptr
        loads.append(block_idx)            # K block -> registers
        ahead = block_idx + distance * w
        if distance > 0 and ahead < e:     # guard: nothing at or past e is touched
            lookups.append(ahead)          # bt[block_idx + w] -> next_k_ptr
            prefetches.append(ahead)
        block_idx += w                     # (compute QK^T happens here)
    return lookups, loads, prefetches
