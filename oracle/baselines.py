"""Baseline verifiers of one level of K draft tokens drawn i.i.d. (WITH replacement) from the draft
distribution: K-SEQ of SpecTr and multi-round rejection sampling of SpecInfer.

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

Both are stated in Sec. 2 (tree-based speculative decoding) and compared with recursive
rejection sampling in the toy example of Sec. 3.1.  With target q, draft p and drafts
x_1..x_K ~ p i.i.d.:

K-SEQ.  For k = 1..K in order, draft x_k is accepted with probability
    min(1, q(x_k) / (gamma p(x_k))),   gamma in [1, K];
the first accepted draft is the output.  If all are rejected the output is drawn from
    Norm[ q - min(p, q / gamma) (1 - (1 - beta)^K) / beta ],   beta = sum_x min(p(x), q(x) / gamma).

Multi-round rejection sampling (one draft model: p^(k) = p for every k).  With q^(1) = q,
draft x_k is accepted with probability min(1, q^(k)(x_k) / p(x_k)) and
    q^(k+1) = Norm[(q^(k) - p)^+];
if all are rejected the output is drawn from q^(K+1).

Readings where the paper is silent: gamma is an argument (SpecTr searches for it; gamma = K is
always admissible); an entry of the K-SEQ residual that comes out negative (possible only for a
gamma that is too small) counts as zero and raises a flag; a stage of the multi-round chain whose
residual has no mass keeps q^(k) and raises a flag (as in recursive rejection sampling); the
acceptance test is the strict U < threshold; the final draw is a Gumbel-max sample.
"""
import numpy as np

from . import philox
from .gumbel_topk import top_k_desc
from .rrs import softmax_row

METHOD_KSEQ = 0
METHOD_MULTIROUND = 1


def kseq_thresholds(q, p, drafts, gamma):
    """(theta [K], residual distribution, flag) of K-SEQ for target q, draft p."""
    q = np.asarray(q, dtype=np.float64)
    p = np.asarray(p, dtype=np.float64)
    K = len(drafts)
    theta = np.array([min(1.0, q[x] / (gamma * p[x])) if p[x] > 0 else 1.0 for x in map(int, drafts)])
    cap = np.minimum(p, q / gamma)
    beta = cap.sum()
    factor = (1.0 - (1.0 - beta) ** K) / beta if beta > 0 else float(K)
    raw = q - cap * factor
    flag = bool(np.any(raw < -1e-15 * np.maximum(q, 1e-300)))
    res = np.maximum(raw, 0.0)
    mass = res.sum()
    if not (mass > 0 and np.isfinite(mass)):
        return theta, q.copy(), True
    return theta, res / mass, flag


def multiround_thresholds(q, p, drafts):
    """(theta [K], last residual q^(K+1), flag) of multi-round rejection sampling."""
    q = np.array(q, dtype=np.float64)
    p = np.asarray(p, dtype=np.float64)
    theta, flag = [], False
    for x in map(int, drafts):
        theta.append(min(1.0, q[x] / p[x]) if p[x] > 0 else 1.0)
        r = np.maximum(q - p, 0.0)
        mass = r.sum()
        if mass > 0 and np.isfinite(mass):
            q = r / mass
        else:
            flag = True
    return np.array(theta), q, flag


def verify_core(target_logits, draft_logits, drafts, method, gamma, uniforms, last_gumbel,
                inv_temperature=1.0):
    """One level.  Returns dict(accepted (index into drafts or -1), token, theta [K], flag,
    final_dist, last_gap)."""
    q = softmax_row(target_logits, inv_temperature)
    p = softmax_row(draft_logits, inv_temperature)
    if method == METHOD_KSEQ:
        theta, final, flag = kseq_thresholds(q, p, drafts, gamma)
    else:
        theta, final, flag = multiround_thresholds(q, p, drafts)
    for k, x in enumerate(drafts):
        if uniforms[k] < theta[k]:
            return dict(accepted=k, token=int(x), theta=theta, flag=False, final_dist=None, last_gap=np.inf)
    with np.errstate(divide="ignore"):
        score = np.log(final) + np.asarray(last_gumbel, dtype=np.float64)
    best = top_k_desc(score, 2)
    gap = float(score[best[0]] - score[best[1]]) if len(best) > 1 else np.inf
    return dict(accepted=-1, token=int(best[0]), theta=theta, flag=flag, final_dist=final, last_gap=gap)


def verify(target_logits, draft_logits, drafts, method, gamma=1.0, inv_temperature=1.0,
           seq_id=None, node_id=None, seed=0, step=0):
    """Batched: target_logits, draft_logits [R,V]; drafts [R,K] tokens.  The uniform of draft k of
    row r is Philox stream tag 1 at (seq_id[r], node_id[r], vocab index k); the final Gumbel noise
    stream tag 2 at (seq_id[r], node_id[r], .).  Defaults: seq 0, node = row index.
    Returns dict(accepted [R], token [R], theta [R,K], flags [R], near_tie [R], last_gap [R])."""
    target_logits = np.asarray(target_logits)
    draft_logits = np.asarray(draft_logits)
    drafts = np.asarray(drafts)
    R, V = target_logits.shape
    K = drafts.shape[1]
    seq_id = np.zeros(R, dtype=np.int64) if seq_id is None else np.asarray(seq_id)
    node_id = np.arange(R, dtype=np.int64) if node_id is None else np.asarray(node_id)
    acc = np.full(R, -1, dtype=np.int64)
    tok = np.zeros(R, dtype=np.int64)
    theta = np.zeros((R, K))
    flags = np.zeros(R, dtype=bool)
    near = np.zeros(R, dtype=bool)
    gaps = np.full(R, np.inf)
    uni = np.zeros((R, K))
    for r in range(R):
        s, n = int(seq_id[r]), int(node_id[r])
        u = philox.uniform_from_word(philox.words(seed, step, philox.TAG_ACCEPT_UNIFORM, s, n, np.arange(K)))
        g = philox.gumbel_row(seed, step, philox.TAG_LAST_GUMBEL, s, n, V)
        res = verify_core(target_logits[r], draft_logits[r], drafts[r], method, gamma, u, g, inv_temperature)
        acc[r], tok[r], theta[r], flags[r], gaps[r] = res["accepted"], res["token"], res["theta"], res["flag"], res["last_gap"]
        uni[r] = u
        upto = K if res["accepted"] < 0 else res["accepted"] + 1
        near[r] = bool(np.any(np.abs(u[:upto] - res["theta"][:upto]) < 1e-5))
    return dict(accepted=acc, token=tok, theta=theta, flags=flags, near_tie=near, last_gap=gaps, uniforms=uni)
