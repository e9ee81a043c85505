"""Recursive rejection sampling: one sibling group, and the walk over a tree.

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

Single group (Sec. 3.1; Eqs. (1)-(4); Alg. 1).  K draft tokens x_1..x_K are
drawn in order without replacement from the draft distribution p, i.e.
p^(k) = p with x_1..x_{k-1} zeroed and renormalised.  With q^(1) = q:
  Theta^(k) = min(1, q^(k)(x_k) / p^(k)(x_k))                      Eq. (3)
  q^(k+1)   = Norm[(q^(k) - p^(k))^+]                              Eq. (2)
Token x_k is accepted with probability Theta^(k) given all earlier ones were
rejected; if all K are rejected the output is drawn from q^(K+1)   Eq. (4).

Tree walk (Sec. 3.2.2, verification; Alg. 6).  Start at the root.  The
children of the current node, in stored order (decreasing perturbed score),
form one sibling group verified with p = draft(.|node), q = target(.|node).
The first accepted child becomes the current node; if all are rejected the
last token is drawn from the final residual; a node without children draws
the last token from the target distribution itself.  The last token is a
Gumbel-max sample (Alg. 6, last lines).

Readings of Alg. 6 (its listing has index slips): the inner loop runs over
the positions j of the level whose parent id equals the current node; the
token zeroed in the draft distribution is the rejected token x_d; accepted
tokens and accepted node ids are separate lists; the acceptance test is the
strict U < Theta.  If a residual mass is not positive (impossible in exact
arithmetic after a genuine rejection) q^(k) is kept and a flag is raised.

Tree layout: level-ordered nodes, node 0 = root, parent[i] < i, parent[0] = -1,
tokens[i] = draft token of node i (tokens[0] unused).  Logit row i holds the
model's next-token logits *after* the sequence ending in node i.
"""
import numpy as np

from . import philox
from .gumbel_topk import log_softmax_rows, top_k_desc

MODE_PATH = 0
MODE_ALL_GROUPS = 1


def softmax_row(logits, inv_temperature=1.0):
    phi, _ = log_softmax_rows(np.asarray(logits).reshape(1, -1), inv_temperature)
    return np.exp(phi[0])


def sibling_chain(q, p, tokens):
    """Thresholds and residuals of one sibling group (Eqs. (2), (3)).

    q, p: target / draft probability vectors; tokens: x_1..x_K (distinct).
    Returns (theta [K], residuals [K+1 arrays: q^(1)..q^(K+1)], degenerate [K]
    booleans: stage k had no positive residual mass, so q^(k+1) = q^(k)).
    """
    q = np.array(q, dtype=np.float64)
    p = np.array(p, dtype=np.float64)
    thetas, residuals, degenerate = [], [q.copy()], []
    for x in tokens:
        x = int(x)
        thetas.append(min(1.0, q[x] / p[x]) if p[x] > 0 else 1.0)
        r = np.maximum(q - p, 0.0)
        mass = r.sum()
        ok = bool(np.isfinite(mass) and mass > 0)
        degenerate.append(not ok)
        if ok:
            q = r / mass               # else keep q^(k)
        p = p.copy()
        p[x] = 0.0
        mass_p = p.sum()
        if mass_p > 0:
            p = p / mass_p
        residuals.append(q.copy())
    return np.array(thetas), residuals, np.array(degenerate, dtype=bool)


def children_of(parent, n_nodes, node):
    return [j for j in range(1, int(n_nodes)) if int(parent[j]) == node]


def recursive_reject_core(target_logits, draft_logits, tokens, parent, n_nodes,
                          uniforms, last_gumbel, inv_temperature=1.0,
                          mode=MODE_PATH):
    """Alg. 6 for one sequence with the random numbers passed in.

    target_logits, draft_logits [N,V]; tokens, parent [N]; uniforms [N]
    (uniforms[j] decides node j); last_gumbel(node) -> [V] Gumbel noise used
    if the last token is drawn at `node`.
    Returns dict: accepted_nodes, accepted_tokens, last_token, final_node,
    final_dist (probabilities the last token is drawn from), theta [N]
    (NaN where not computed), flag (degenerate residual met),
    last_gap (top-1 minus top-2 of the final perturbed scores).
    """
    n = int(n_nodes)
    theta = np.full(len(tokens), np.nan)
    flag = False
    if mode == MODE_ALL_GROUPS:
        for node in range(n):
            kids = children_of(parent, n, node)
            if kids:
                th, _, dg = sibling_chain(
                    softmax_row(target_logits[node], inv_temperature),
                    softmax_row(draft_logits[node], inv_temperature),
                    [tokens[j] for j in kids])
                theta[kids] = th
    cur, accepted = 0, []
    while True:
        q = softmax_row(target_logits[cur], inv_temperature)
        kids = children_of(parent, n, cur)
        if not kids:
            final = q
            break
        p = softmax_row(draft_logits[cur], inv_temperature)
        th, residuals, dg = sibling_chain(q, p, [tokens[j] for j in kids])
        took = None
        for k, j in enumerate(kids):
            theta[j] = th[k]
            if uniforms[j] < th[k]:
                took = j
                flag = flag or bool(np.any(dg[:k]))   # residuals behind theta[k]
                break
        if took is None:
            final = residuals[len(kids)]
            flag = flag or bool(np.any(dg))   # every stage's residual was used
            break
        accepted.append(took)
        cur = took
    with np.errstate(divide="ignore"):
        score = np.log(final) + np.asarray(last_gumbel(cur), dtype=np.float64)
    best = top_k_desc(score, 2)
    gap = float(score[best[0]] - score[best[1]]) if len(best) > 1 else np.inf
    return dict(accepted_nodes=np.array(accepted, dtype=np.int64),
                accepted_tokens=np.array([tokens[j] for j in accepted], dtype=np.int64),
                last_token=int(best[0]), final_node=cur, final_dist=final,
                theta=theta, flag=flag, last_gap=gap)


def recursive_reject(target_logits, draft_logits, tokens, parent, n_nodes,
                     inv_temperature=1.0, mode=MODE_PATH, seq_id=None,
                     seed=0, step=0, depth_max=None):
    """Batched Alg. 6 with Philox randomness.

    target_logits, draft_logits [B,N,V]; tokens, parent [B,N]; n_nodes [B].
    Uniform for node j of sequence b: stream tag 1 at (seq_id[b], j, vocab 0);
    last-token Gumbel at node c: stream tag 2 at (seq_id[b], c, .).
    Returns dict of arrays: accepted_nodes [B,depth_max] (-1 pad),
    accepted_tokens, n_accepted, last_token, final_node, theta, uniforms,
    flags, near_tie (|u - theta| < 1e-5 on a decided node), last_gap.
    """
    target_logits = np.asarray(target_logits)
    draft_logits = np.asarray(draft_logits)
    B, N, V = target_logits.shape
    seq_id = np.arange(B) if seq_id is None else np.asarray(seq_id)
    depth_max = N if depth_max is None else depth_max
    acc = np.full((B, depth_max), -1, dtype=np.int64)
    acc_tok = np.full((B, depth_max), -1, dtype=np.int64)
    n_acc = np.zeros(B, dtype=np.int64)
    last = np.zeros(B, dtype=np.int64)
    final_node = np.zeros(B, dtype=np.int64)
    theta = np.full((B, N), np.nan)
    uni = np.zeros((B, N))
    flags = np.zeros(B, dtype=bool)
    near = np.zeros(B, dtype=bool)
    gaps = np.zeros(B)
    for b in range(B):
        s = int(seq_id[b])
        u = philox.uniform_from_word(philox.words(
            seed, step, philox.TAG_ACCEPT_UNIFORM, s, np.arange(N), 0))
        r = recursive_reject_core(
            target_logits[b], draft_logits[b], tokens[b], parent[b], n_nodes[b], u,
            lambda node: philox.gumbel_row(seed, step, philox.TAG_LAST_GUMBEL, s, node, V),
            inv_temperature, mode)
        k = len(r["accepted_nodes"])
        acc[b, :k], acc_tok[b, :k], n_acc[b] = r["accepted_nodes"], r["accepted_tokens"], k
        last[b], final_node[b] = r["last_token"], r["final_node"]
        theta[b], uni[b], flags[b], gaps[b] = r["theta"], u, r["flag"], r["last_gap"]
        # decided nodes: children groups visited by the walk
        cur = 0
        for j in list(r["accepted_nodes"]) + [None]:
            for c in children_of(parent[b], n_nodes[b], cur):
                if abs(u[c] - theta[b, c]) < 1e-5:
                    near[b] = True
                if c == j:
                    break
            if j is None:
                break
            cur = int(j)
    return dict(accepted_nodes=acc, accepted_tokens=acc_tok, n_accepted=n_acc,
                last_token=last, final_node=final_node, theta=theta, uniforms=uni,
                flags=flags, near_tie=near, last_gap=gaps)
