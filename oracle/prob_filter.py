"""Probability filtering of a next-token distribution: top-k and nucleus (top-p).

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

The experiments sample the instruction-following task with nucleus (top-p)
sampling, p = 0.95, at temperature 1 (Sec. 4, experiment setup), and the
samplers drop candidates whose log-probability is -inf "when probability
filtering methods (e.g. top-p, top-k) were applied" (last step of Alg. 4 and
of Alg. 9).  Filtering therefore acts on the logits of both models before
drafting and verification: entries outside the kept set become -inf, and the
softmax that every later step takes renormalises over what is left.

Definitions used (the paper cites the nucleus-sampling paper and prints none):
* top-k keeps the k most probable entries;
* top-p keeps the smallest set of most probable entries whose probability mass
  reaches p;
* entries as probable as the least probable kept entry are kept as well (a
  rule that does not depend on how equal values happen to be ordered);
* when both are given, top-k acts first and top-p acts on the distribution
  renormalised over the top-k set;
* entries that are -inf on input stay -inf and never count.
"""
import numpy as np


def _softmax64(z):
    m = np.max(z)
    e = np.exp(z - m)
    return e / e.sum()


def filter_row(z, inv_temperature=1.0, top_k=0, top_p=1.0):
    """One row of logits -> (filtered logits, margin).

    `margin` is how far the deciding comparisons were from flipping: the smallest of the gap
    between the top-p target and the cumulative masses on either side of the cut, and the
    relative gap between the least probable kept entry and the most probable dropped one
    (for either filter; inf when a filter is off or nothing is dropped).  A reader that works
    in lower precision may see such a pair as equally probable and, by the rule above, keep
    both.
    """
    z = np.asarray(z)
    x = z.astype(np.float64) * np.float64(np.float32(inv_temperature))
    keep = np.isfinite(x)
    margin = np.inf
    if not keep.any():
        return np.full(z.shape, -np.inf, dtype=z.dtype), margin
    prob = np.where(keep, _softmax64(np.where(keep, x, -np.inf)), 0.0)
    if top_k and top_k < int(keep.sum()):
        srt = np.sort(prob[keep])[::-1]
        kth = srt[top_k - 1]
        dropped = srt[srt < kth]         # (entries tied with the k-th are kept, not dropped)
        if dropped.size:
            margin = min(margin, (kth - dropped[0]) / kth)
        keep &= prob >= kth
        prob = np.where(keep, prob, 0.0)
        prob = prob / prob.sum()
    if top_p < 1.0:
        srt = np.sort(prob[keep])[::-1]
        cum = np.cumsum(srt)
        i = int(np.searchsorted(cum, top_p, side="left"))  # first index with cum >= p
        i = min(i, len(srt) - 1)
        thr = srt[i]
        below = cum[i - 1] if i > 0 else 0.0
        margin = min(margin, cum[i] - top_p, top_p - below)
        dropped = srt[srt < thr]
        if dropped.size:
            margin = min(margin, (thr - dropped[0]) / thr)
        keep &= prob >= thr
    out = np.where(keep, z, np.asarray(-np.inf, dtype=z.dtype))
    return out.astype(z.dtype), float(margin)


def filter_logits(z, inv_temperature=1.0, top_k=0, top_p=1.0):
    """Rows [R, V] -> (filtered [R, V], kept[R], margin[R])."""
    z = np.asarray(z)
    out = np.empty_like(z)
    kept = np.zeros(z.shape[0], dtype=np.int32)
    margin = np.zeros(z.shape[0])
    for r in range(z.shape[0]):
        out[r], margin[r] = filter_row(z[r], inv_temperature, top_k, top_p)
        kept[r] = int(np.isfinite(out[r]).sum())
    return out, kept, margin
