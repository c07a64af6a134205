"""CPU oracle of the block partitioner (App. C.2, Algorithm 2).  TEST INFRASTRUCTURE ONLY.

Plain Python, in the order of the algorithm.  Units are the structural candidates in forward
order; unit j has n_j parameters and a normalised diagnostic vector z_j.  The steps the paper
leaves open are read as follows (the same readings bind the library):

  * statistics of a temporary block = parameter-weighted mean of its units' vectors,
    accumulated in unit order;
  * Delta(U_a, U_b) = max_k w_k |z_a,k - z_b,k|;
  * tau = upper quartile (q = 0.75, linear interpolation between order statistics) of
    Delta over all pairs of candidate units; 0 when there is a single unit;
  * n_min = alpha * |Theta|;
  * minimum-size filtering: while a temporary block is smaller than n_min (and more than one
    block is left) the first such block is merged into the adjacent block with the smaller
    Delta to it; on a tie the smaller neighbour, then the left one;
  * block formation: a boundary between adjacent temporary blocks is kept when their Delta
    exceeds tau and both have at least n_min parameters; otherwise they end up in one block;
  * post-processing, split: a formed block made of several temporary blocks is cut at the
    internal boundary where the two sides' statistics differ most, if that difference exceeds
    tau and both sides have at least n_min parameters; the parts are examined again;
  * post-processing, re-merge: the minimum-size rule once more on the final blocks.

parity unpinned against the paper: it prints no partition.  Pinned by hand-worked cases and
invariants (tests/test_partition.py).
"""


def _stats(units, z, numel):
    """Parameter-weighted mean vector of a run of unit indices, and its size."""
    K = len(z[0])
    acc = [0.0] * K
    size = 0
    for j in units:
        size += numel[j]
        for k in range(K):
            acc[k] += float(numel[j]) * z[j][k]
    return [a / float(size) for a in acc], size


def _delta(za, zb, w):
    d = 0.0
    for k in range(len(za)):
        x = w[k] * abs(za[k] - zb[k])
        if x > d:
            d = x
    return d


def _upper_quartile(vals):
    if not vals:
        return 0.0
    s = sorted(vals)
    pos = 0.75 * (len(s) - 1)
    lo = int(pos)
    hi = min(lo + 1, len(s) - 1)
    return s[lo] + (pos - lo) * (s[hi] - s[lo])


def _merge_small(blocks, z, numel, w, n_min):
    """blocks: list of lists of unit indices (contiguous, in order)."""
    while len(blocks) > 1:
        small = None
        for i, b in enumerate(blocks):
            if _stats(b, z, numel)[1] < n_min:
                small = i
                break
        if small is None:
            break
        zs, _ = _stats(blocks[small], z, numel)
        cands = []
        for nb in (small - 1, small + 1):
            if 0 <= nb < len(blocks):
                zn, sn = _stats(blocks[nb], z, numel)
                cands.append((_delta(zs, zn, w), sn, nb))
        cands.sort(key=lambda c: (c[0], c[1], c[2]))
        nb = cands[0][2]
        lo, hi = min(small, nb), max(small, nb)
        blocks[lo:hi + 1] = [blocks[lo] + blocks[hi]]
    return blocks


def _split(temp_blocks, z, numel, w, tau, n_min):
    """temp_blocks: the temporary blocks of one formed block. Returns a list of lists of temporary blocks."""
    if len(temp_blocks) < 2:
        return [temp_blocks]
    best, at = -1.0, None
    for p in range(1, len(temp_blocks)):
        left = [u for b in temp_blocks[:p] for u in b]
        right = [u for b in temp_blocks[p:] for u in b]
        zl, sl = _stats(left, z, numel)
        zr, sr = _stats(right, z, numel)
        if sl < n_min or sr < n_min:
            continue
        d = _delta(zl, zr, w)
        if d > best:
            best, at = d, p
    if at is None or not best > tau:
        return [temp_blocks]
    return _split(temp_blocks[:at], z, numel, w, tau, n_min) + _split(temp_blocks[at:], z, numel, w, tau, n_min)


def partition(numel, z, weights=None, alpha=0.01):
    """-> (block id per unit, number of blocks, tau)."""
    m = len(numel)
    K = len(z[0])
    w = [1.0] * K if weights is None else [float(x) for x in weights]
    z = [[float(x) for x in row] for row in z]
    total = sum(int(n) for n in numel)
    n_min = alpha * float(total)

    # statistic difference over all pairs of candidate units; tau = their upper quartile
    pair = []
    for a in range(m):
        for b in range(a + 1, m):
            pair.append(_delta(z[a], z[b], w))
    tau = _upper_quartile(pair)

    # minimum-size filtering on the candidate units
    temp = _merge_small([[j] for j in range(m)], z, numel, w, n_min)

    # block formation over adjacent temporary blocks
    formed = [[temp[0]]]
    for i in range(1, len(temp)):
        za, sa = _stats(temp[i - 1], z, numel)
        zb, sb = _stats(temp[i], z, numel)
        if _delta(za, zb, w) > tau and sa >= n_min and sb >= n_min:
            formed.append([temp[i]])
        else:
            formed[-1].append(temp[i])

    # post-processing: split, then re-merge what is still too small
    final = []
    for f in formed:
        for part in _split(f, z, numel, w, tau, n_min):
            final.append([u for b in part for u in b])
    final = _merge_small(final, z, numel, w, n_min)

    ids = [0] * m
    for bi, b in enumerate(final):
        for u in b:
            ids[u] = bi
    return ids, len(final), tau
