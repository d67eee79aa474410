"""Oracle of the transfer schedule: parameter / gradient tensors packed into a stage's M data-transfer windows.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Paper Sec. 4.2, "Scheduling parameter transfers": the tensors are sorted by size in descending order and each is given
to the window whose assigned bytes are smallest so far (longest-processing-time-first list scheduling, Graham 1969);
very large tensors are split into smaller chunks first.  The paper fixes neither the chunk size nor the tie-breaks; the
reading used here: a tensor above max_piece is cut into ceil(bytes / max_piece) equal pieces rounded up to 256 bytes
(the last piece takes the remainder); equal sizes keep tensor order, then offset order; equal loads go to the lower
window.
"""


def split_items(item_bytes, max_piece):
    pieces = []
    for i, b in enumerate(item_bytes):
        if b == 0:
            continue
        n = -(-b // max_piece)
        sz = -(-b // n)
        sz = -(-sz // 256) * 256
        off = 0
        while off < b:
            pieces.append((i, off, min(sz, b - off)))
            off += sz
    return pieces


def lpt(item_bytes, n_windows, max_piece):
    """Returns [(item, window, offset, bytes)] in assignment order."""
    pieces = sorted(split_items(item_bytes, max_piece), key=lambda p: (-p[2], p[0], p[1]))
    load = [0] * n_windows
    out = []
    for item, off, nbytes in pieces:
        w = min(range(n_windows), key=lambda k: (load[k], k))
        load[w] += nbytes
        out.append((item, w, off, nbytes))
    return out


def makespan(plan, n_windows):
    load = [0] * n_windows
    for _, w, _, nbytes in plan:
        load[w] += nbytes
    return max(load)


def optimal_makespan(sizes, n_windows):
    """Brute force over every assignment (tiny inputs only)."""
    best = [sum(sizes)]

    def rec(i, load):
        if max(load) >= best[0]:
            return
        if i == len(sizes):
            best[0] = max(load)
            return
        seen = set()
        for w in range(n_windows):
            if load[w] in seen:
                continue
            seen.add(load[w])
            load[w] += sizes[i]
            rec(i + 1, load)
            load[w] -= sizes[i]

    rec(0, [0] * n_windows)
    return best[0]
