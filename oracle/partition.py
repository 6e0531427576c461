"""Oracle for the message partition between the device path and the host path.

TEST INFRASTRUCTURE, NOT THE PRODUCT.  Shares no code with the HIP library.

The paper's Communicator divides each collective's payload over the paths in
proportion to the share vector and runs all paths at once (Design, first
paragraphs; Section "Two-Stage Load Balancing Strategy").  With two paths the
partition is one cut point.  The paper does not say where a path's part lies
inside the message or how it is rounded; the reading here:

* the device path takes the head [0, split), the host path the tail
  [split, count);
* with host share u out of `total` units the host path is owed
  floor(count * u / total) elements; the cut is then moved down to a multiple
  of `align` elements, so the host part never shrinks by rounding;
* u == 0, or a message shorter than `min_count` elements, is not split
  (split == count); u == total gives split == 0;
* a non-zero share always yields a non-empty host part: if rounding left it
  empty, it gets one alignment quantum.
"""


def partition(count, host_units, total=10000, align=2048, min_count=32768):
    if host_units < 0 or host_units > total:
        raise ValueError("host share out of range")
    if host_units == 0 or count < min_count or count < align:
        return count
    if host_units == total:
        return 0
    owed = (count * host_units) // total
    split = ((count - owed) // align) * align
    if split == count:
        split = count - align
    return split


def partition_paths(count, units, total=10000, align=2048, min_count=32768):
    """Several auxiliary paths.  units[p] is path p's share (units[0], the
    primary path's, is not used: it gets what is left).  Returns the list
    `start` of len(units) + 1 offsets: path p carries [start[p], start[p+1]).

    Reading: the pieces are laid out in path order; they are cut from the end
    of the message backwards, each by the two-path rule applied to what is
    still unassigned in front of it: owed = floor(count * units[p] / total)
    elements, the piece's start rounded down to a multiple of `align` (not
    below 0), one alignment quantum at least for a non-zero share while
    anything is left.  Messages shorter than `min_count` or `align` are not
    split."""
    if sum(units[1:]) > total or min(units) < 0:
        raise ValueError("shares out of range")
    n = len(units)
    start = [0] * (n + 1)
    start[n] = count
    end = count
    for p in range(n - 1, 0, -1):
        s = end
        if units[p] > 0 and count >= min_count and count >= align:
            owed = (count * units[p]) // total
            s = ((end - owed) // align) * align if end > owed else 0
            if s == end:                       # rounding left the piece empty
                s = ((end - 1) // align) * align if end >= align else 0
        start[p] = s
        end = s
    return start
