"""Gumbel-Top-k sampling without replacement (the RSD-C sampler).

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

Follows Sec. 3.2.1 (RSD-C), Eqs. (5)-(7) and Alg. 4 (SampleWithGumbelTopK):
  phi       = log-softmax(logits / T)                      Eq. (5)
  phi_tilde = phi + G,  G i.i.d. standard Gumbel           Eq. (6)
  tokens    = the k entries with the largest phi_tilde,
              in decreasing order of phi_tilde             Eq. (7)
Entries whose log-probability is -inf are never returned (last step of
Alg. 4), so fewer than k tokens may come back.

Readings where the paper is silent: exact ties in phi_tilde go to the lower
token index; the temperature divides the logits before the softmax.
"""
import numpy as np

from . import philox


def log_softmax_rows(logits, inv_temperature=1.0):
    """(phi, lse) in fp64: phi = z/T - lse, lse = log sum exp(z/T)."""
    z = np.asarray(logits, dtype=np.float64) * float(inv_temperature)
    z = np.atleast_2d(z)
    m = np.max(z, axis=-1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    lse = m + np.log(np.sum(np.exp(z - m), axis=-1, keepdims=True))
    return z - lse, lse[:, 0]


def top_k_desc(values, k):
    """Indices of the k largest finite-or-+inf entries, decreasing value,
    lower index first among equals; -inf and NaN entries are skipped."""
    v = np.asarray(values, dtype=np.float64)
    idx = np.arange(v.shape[0])
    keep = v > -np.inf            # False for -inf and NaN
    idx = idx[keep]
    order = np.lexsort((idx, -v[idx]))   # primary: -value, secondary: index
    return idx[order[:k]]


def gumbel_topk_from_noise(logits, gumbel, k_per_row, inv_temperature=1.0):
    """Alg. 4 with the Gumbel matrix passed in.

    logits [R,V], gumbel [R,V], k_per_row [R] ints.
    Returns per-row lists: tokens, perturbed log-probs, log-probs; and lse[R].
    """
    phi, lse = log_softmax_rows(logits, inv_temperature)
    phi_tilde = phi + np.asarray(gumbel, dtype=np.float64)
    toks, pert, logp = [], [], []
    for r in range(phi.shape[0]):
        sel = top_k_desc(phi_tilde[r], int(k_per_row[r]))
        toks.append(sel.astype(np.int64))
        pert.append(phi_tilde[r, sel])
        logp.append(phi[r, sel])
    return toks, pert, logp, lse


def gumbel_topk(logits, k_max, k_per_row=None, inv_temperature=1.0,
                seq_id=None, node_id=None, seed=0, step=0):
    """Alg. 4 with Philox noise (stream tag 0).

    Row r uses counter coordinates (seq_id[r], node_id[r]); defaults are
    seq 0 and node = row index.  Output arrays are padded to k_max with
    token -1, perturbed/logprob -inf; count[r] gives the valid length.
    """
    logits = np.atleast_2d(np.asarray(logits))
    R, V = logits.shape
    k_per_row = (np.full(R, k_max, dtype=np.int64) if k_per_row is None
                 else np.asarray(k_per_row, dtype=np.int64))
    seq_id = np.zeros(R, dtype=np.int64) if seq_id is None else np.asarray(seq_id)
    node_id = np.arange(R, dtype=np.int64) if node_id is None else np.asarray(node_id)
    g = np.stack([philox.gumbel_row(seed, step, philox.TAG_DRAFT_GUMBEL,
                                    int(seq_id[r]), int(node_id[r]), V)
                  for r in range(R)])
    toks, pert, logp, lse = gumbel_topk_from_noise(
        logits, g, np.minimum(k_per_row, k_max), inv_temperature)
    tokens = np.full((R, k_max), -1, dtype=np.int64)
    perturbed = np.full((R, k_max), -np.inf)
    logprob = np.full((R, k_max), -np.inf)
    count = np.zeros(R, dtype=np.int64)
    for r in range(R):
        n = len(toks[r])
        tokens[r, :n], perturbed[r, :n], logprob[r, :n] = toks[r], pert[r], logp[r]
        count[r] = n
    return dict(tokens=tokens, perturbed=perturbed, logprob=logprob,
                lse=lse, count=count)


def near_tie_rows(logits, k_per_row, inv_temperature, seq_id, node_id,
                  seed, step, tol=1e-5):
    """Rows whose selection could flip under a perturbation < tol: some
    adjacent gap among the top (k+1) perturbed values is below tol."""
    logits = np.atleast_2d(np.asarray(logits))
    R, V = logits.shape
    out = np.zeros(R, dtype=bool)
    phi, _ = log_softmax_rows(logits, inv_temperature)
    for r in range(R):
        g = philox.gumbel_row(seed, step, philox.TAG_DRAFT_GUMBEL,
                              int(seq_id[r]), int(node_id[r]), V)
        pt = phi[r] + g
        k = int(k_per_row[r])
        top = np.sort(pt[pt > -np.inf])[::-1][:k + 1]
        out[r] = bool(np.any(-np.diff(top) < tol))
    return out
