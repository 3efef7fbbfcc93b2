"""Plain CPU oracle of the layer-wise bit-width assigners (paper Sec. "Layer-wise
Adaptive Quantization": the sort-and-interpolate heuristic and Algorithm 1, the
k-means based one).  TEST INFRASTRUCTURE, like the rest of this package.

The paper fixes the structure (2-D points (size, norm) per layer, k-means into
k = |B| clusters, centroids sorted by norm - size, bit-widths mapped onto that
order) and leaves the details open.  Readings used here, step by step:

  points      layers with bits_in != 0 and size > 0 take part (the others keep 0:
              filtered layers travel uncompressed).  Each axis is scaled to [0, 1]
              by its minimum and maximum over those layers (an axis with no spread
              becomes 0), so that "norm - size" compares like with like.
  start       points are sorted by key = y - x (ties: layer order); centroid c
              starts at the point of rank floor((c + 1/2) * M / k) in that order.
  iteration   Lloyd: every point goes to its nearest centroid (squared Euclidean
              distance, ties to the lowest index); a centroid becomes the mean of
              its points (sums taken in layer order; an empty cluster keeps its
              centroid); stop when no point changes cluster or after max_iter rounds.
  mapping     non-empty clusters are ranked by centroid y - x, ascending (ties: lower
              index first); rank r of m gets candidates[round_half_up(r*(k-1)/(m-1))]
              (m == 1: the largest candidate), candidates ascending.  So large
              layers with small gradients get the fewest bits.
  fewer points than clusters: every point is its own cluster (same mapping).

The linear heuristic: layers sorted by norm / size ascending (ties: layer order);
rank r of M gets candidates[floor(r * k / M)].
"""
from __future__ import annotations

import numpy as np


def _active(sizes, bits_in):
    return [l for l in range(len(sizes)) if bits_in[l] != 0 and sizes[l] > 0]


def _unit_axis(v):
    lo, hi = min(v), max(v)
    if not hi > lo:
        return [0.0 for _ in v]
    return [(t - lo) / (hi - lo) for t in v]


def _map_rank(r, m, cands):
    k = len(cands)
    if m == 1:
        return cands[k - 1]
    return cands[(2 * r * (k - 1) + (m - 1)) // (2 * (m - 1))]


def kmeans_bits(sizes, norms, bits_in, candidates, max_iter=100, details=False):
    sizes = [float(s) for s in sizes]
    norms = [float(t) for t in norms]
    cands = sorted(int(c) for c in candidates)
    k = len(cands)
    out = [0] * len(sizes)
    act = _active(sizes, bits_in)
    M = len(act)
    if M == 0 or k == 0:
        return (np.array(out, np.uint8), None) if details else np.array(out, np.uint8)
    xs = _unit_axis([sizes[l] for l in act])
    ys = _unit_axis([norms[l] for l in act])
    key = [ys[i] - xs[i] for i in range(M)]
    order = sorted(range(M), key=lambda i: (key[i], i))
    if M <= k:
        label = [0] * M
        for r, i in enumerate(order):
            label[i] = r
        cx, cy = [xs[i] for i in order], [ys[i] for i in order]
        kk = M
    else:
        kk = k
        start = [order[((2 * c + 1) * M) // (2 * k)] for c in range(k)]
        cx, cy = [xs[i] for i in start], [ys[i] for i in start]
        label = [-1] * M
        for _ in range(max_iter):
            changed = False
            for i in range(M):
                best, bd = 0, None
                for c in range(kk):
                    dx, dy = xs[i] - cx[c], ys[i] - cy[c]
                    d = dx * dx + dy * dy
                    if bd is None or d < bd:
                        best, bd = c, d
                if best != label[i]:
                    label[i] = best
                    changed = True
            if not changed:
                break
            for c in range(kk):
                sx = sy = 0.0
                cnt = 0
                for i in range(M):
                    if label[i] == c:
                        sx += xs[i]
                        sy += ys[i]
                        cnt += 1
                if cnt:
                    cx[c], cy[c] = sx / cnt, sy / cnt
    used = sorted({label[i] for i in range(M)}, key=lambda c: (cy[c] - cx[c], c))
    rank = {c: r for r, c in enumerate(used)}
    for i, l in enumerate(act):
        out[l] = _map_rank(rank[label[i]], len(used), cands)
    res = np.array(out, np.uint8)
    if details:
        return res, {"x": xs, "y": ys, "label": label, "cx": cx, "cy": cy, "active": act}
    return res


def linear_bits(sizes, norms, bits_in, candidates):
    cands = sorted(int(c) for c in candidates)
    k = len(cands)
    out = [0] * len(sizes)
    act = _active(sizes, bits_in)
    M = len(act)
    if M == 0 or k == 0:
        return np.array(out, np.uint8)
    ratio = {l: float(norms[l]) / float(sizes[l]) for l in act}
    order = sorted(act, key=lambda l: (ratio[l], l))
    for r, l in enumerate(order):
        out[l] = cands[(r * k) // M]
    return np.array(out, np.uint8)


def buckets_from_bits(bits, width_candidates, bucket_candidates):
    """Bucket size per layer from the widths an assigner chose.

    The section maps bit-widths and bucket sizes to the layers linearly over the same order of
    layers; it prints no rule for the bucket sizes.  Reading used: the position of a layer's
    width among the ascending width candidates decides, linearly, its position among the
    DESCENDING bucket candidates, so the layers that get the fewest bits also get the longest
    buckets (both choices compress more): width number i of k takes bucket number
    round_half_up(i * (kb - 1) / (k - 1)) of kb (k = 1: the longest bucket).  Layers with width
    0 (uncompressed) take the longest bucket, which nothing uses.
    """
    widths = sorted(int(c) for c in width_candidates)
    sizes = sorted((int(c) for c in bucket_candidates), reverse=True)
    k, kb = len(widths), len(sizes)
    out = []
    for b in bits:
        b = int(b)
        if b == 0:
            out.append(sizes[0])
            continue
        i = widths.index(b)               # an assigned width is one of the candidates
        j = 0 if k == 1 else (2 * i * (kb - 1) + (k - 1)) // (2 * (k - 1))
        out.append(sizes[j])
    return np.array(out, np.int32)
