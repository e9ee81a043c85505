"""One Stochastic Beam Search expansion step (the RSD-S sampler).

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

Follows Sec. 3.2.1 (RSD-S), Eqs. (10)-(12) and Alg. 9
(SampleWithStochasticBeam), in the algorithm's order:
  1. Phi       = log-softmax(logits/T) + Sigma (parent sum log-prob per row)
  2. G         ~ i.i.d. standard Gumbel
  3. Phi_tilde = Phi + G
  4. Z         = row-wise max of Phi_tilde
  5. psi       = T(Gamma, Phi_tilde) = -log(e^-Gamma - e^-Z + e^-Phi_tilde)   Eq. (11)
  6. top-W over all (parent row, token) pairs by psi, decreasing              Eq. (12)
  7. Sigma'    = Phi[parent, token],  Gamma' = psi[parent, token]

Step 5 is evaluated in the algebraically equal form
  psi = Gamma - softplus(v),  v = Gamma - Phi_tilde + log(1 - exp(Phi_tilde - Z)),
which stays finite when the three exponentials of Eq. (11) differ by hundreds
of orders of magnitude; at the row argmax v = -inf and psi = Gamma exactly.

Readings: Alg. 9's last-but-one line ranks by psi (its comment and Eq. (12)
say so, although the printed argument is the perturbed matrix); the root beam
has Sigma = Gamma = 0 (Alg. 8); exact ties go to the lower parent row, then
the lower token; entries with -inf log-probability are dropped.
"""
import numpy as np

from . import philox
from .gumbel_topk import log_softmax_rows


def truncated_gumbel(gamma, phi_tilde, z):
    """T(gamma, phi_tilde) of Eq. (11) with row maximum z, stable form."""
    phi_tilde = np.asarray(phi_tilde, dtype=np.float64)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        d = phi_tilde - z                       # <= 0
        # log(1 - e^d): expm1 near d = 0, log1p(-e^d) for very negative d
        log1m = np.where(d > -np.log(2.0), np.log(-np.expm1(d)), np.log1p(-np.exp(d)))
        log1m = np.where(d < 0, log1m, -np.inf)
        v = gamma - phi_tilde + log1m
        softplus = np.maximum(v, 0.0) + np.log1p(np.exp(-np.abs(v)))
        softplus = np.where(np.isneginf(v), 0.0, softplus)
        psi = gamma - softplus
    return np.where(np.isneginf(phi_tilde), -np.inf, psi)


def sbs_step_from_noise(logits, sum_logprob, trunc_gumbel, gumbel, width,
                        inv_temperature=1.0):
    """Alg. 9 for one sequence with the Gumbel matrix passed in.

    logits [n,V] (one row per live beam entry), sum_logprob [n], trunc_gumbel [n],
    gumbel [n,V].  Returns dict(tokens, parent, sum_logprob, trunc_gumbel, perturbed, lse,
    psi_all); perturbed = Phi_tilde of the selected pairs (Eq. (11) turns an error e in it into
    e * exp(psi - Phi_tilde) in psi, which a comparison in lower precision has to allow for).
    """
    logits = np.atleast_2d(np.asarray(logits))
    n, V = logits.shape
    sigma = np.asarray(sum_logprob, dtype=np.float64).reshape(n, 1)
    gamma = np.asarray(trunc_gumbel, dtype=np.float64).reshape(n, 1)
    phi_tok, lse = log_softmax_rows(logits, inv_temperature)
    phi = phi_tok + sigma                                        # step 1
    phi_tilde = phi + np.asarray(gumbel, dtype=np.float64)       # steps 2-3
    z = np.max(phi_tilde, axis=1, keepdims=True)                 # step 4
    psi = truncated_gumbel(gamma, phi_tilde, z)                  # step 5
    flat = psi.reshape(-1)                                       # step 6
    idx = np.arange(flat.shape[0])
    keep = flat > -np.inf
    idx = idx[keep]
    order = np.lexsort((idx, -flat[idx]))      # ties: lower row, then lower token
    sel = idx[order[:width]]
    ranked = flat[idx[order[:width + 1]]]
    min_gap = float(np.min(-np.diff(ranked))) if ranked.size > 1 else np.inf
    parent = sel // V
    tokens = sel % V
    return dict(tokens=tokens.astype(np.int64), parent=parent.astype(np.int64),
                sum_logprob=phi[parent, tokens],                 # step 7
                trunc_gumbel=psi[parent, tokens], perturbed=phi_tilde[parent, tokens],
                lse=lse, psi_all=psi, min_gap=min_gap)


def sbs_step(logits, sum_logprob, trunc_gumbel, n_in, width, inv_temperature=1.0,
             seq_id=None, node_id=None, seed=0, step=0):
    """Batched Alg. 9 with Philox noise (stream tag 0).

    logits [B,W_in,V]; sum_logprob, trunc_gumbel [B,W_in]; n_in [B] live rows.
    Row (b, w) draws its noise at counter coordinates (seq_id[b], node_id[b,w]);
    defaults: seq = b, node = w.  Outputs padded to `width` with token/parent -1
    and -inf scores; n_out[b] = number of valid entries; min_gap[b] as in
    sbs_step_from_noise (a reader in lower precision may order or cut differently when it is
    tiny).
    """
    logits = np.asarray(logits)
    B, W_in, V = logits.shape
    seq_id = np.arange(B) if seq_id is None else np.asarray(seq_id)
    node_id = (np.tile(np.arange(W_in), (B, 1)) if node_id is None
               else np.asarray(node_id))
    tokens = np.full((B, width), -1, dtype=np.int64)
    parent = np.full((B, width), -1, dtype=np.int64)
    s_out = np.full((B, width), -np.inf)
    g_out = np.full((B, width), -np.inf)
    p_out = np.full((B, width), -np.inf)
    lse = np.zeros((B, W_in))
    n_out = np.zeros(B, dtype=np.int64)
    min_gap = np.full(B, np.inf)
    for b in range(B):
        n = int(n_in[b])
        if n == 0:
            continue
        g = np.stack([philox.gumbel_row(seed, step, philox.TAG_DRAFT_GUMBEL,
                                        int(seq_id[b]), int(node_id[b, w]), V)
                      for w in range(n)])
        r = sbs_step_from_noise(logits[b, :n], sum_logprob[b, :n],
                                trunc_gumbel[b, :n], g, width, inv_temperature)
        m = len(r["tokens"])
        tokens[b, :m], parent[b, :m] = r["tokens"], r["parent"]
        s_out[b, :m], g_out[b, :m] = r["sum_logprob"], r["trunc_gumbel"]
        p_out[b, :m] = r["perturbed"]
        lse[b, :n] = r["lse"]
        n_out[b] = m
        min_gap[b] = r["min_gap"]
    return dict(tokens=tokens, parent=parent, sum_logprob=s_out,
                trunc_gumbel=g_out, perturbed=p_out, n_out=n_out, lse=lse, min_gap=min_gap)
