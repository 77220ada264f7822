"""CPU oracle for the TSLT hot path -- TEST INFRASTRUCTURE, not product code.

A plain, slow, fp64 NumPy implementation of what the paper's method computes per
position: truncated sampling on the draft logits (Section 3.1, Top-K / Top-rho, the
renormalisation equation), "sparsify-then-sample" (Solution 1, Section 3.2), the
single-candidate verification loop (Algorithm 3), multi-candidate verification
(Algorithm 5, with its residual-update equation) and token-tree verification with the
"new sequence searching" walk (Algorithm 8, tree layout of Section 4.1).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this file.
It shares no code with the HIP path and imports nothing from it.  Everything is a full
sort, a sequential cumulative sum or an elementwise NumPy expression so that it can be
checked against the paper by eye; there is no blocking, fusion or reordering.

Pins (tests/test_oracle_*.py): brute-force order properties, nucleus minimality,
TV(q_hat, q) = sigma (Theorem 1), |beta_hat - beta| <= sigma, K = V against
scipy.special.softmax, exhaustive output-distribution = p checks at V <= 16 for
Algorithm 3 and Algorithm 5, beta^(j) and theta (Section 4.3), N_oracle (Section 2.3),
tree identities (Section 4.1) and the k = <1,..,1> reduction of Algorithm 8 to
Algorithm 3.  Behaviour on real model logits (Section 5 figures) is parity unpinned:
the weights are not available.

Readings of the paper taken here (the paper's print is garbled or silent):
  * renormalisation: q_hat(x) = q(x) / sum_{v in V'} q(v) for x in V', 0 otherwise
    (the printed equation has its two cases swapped; proof step (a) of Theorem 1
    confirms this reading);
  * acceptance test: u < min(1, p(x) / q_hat(x)) (Algorithm 3 prints the ratio
    inverted; Algorithm 5 and Lemma 1 have it this way), strict "<";
  * Top-rho: the smallest prefix of the descending order whose mass is >= rho;
  * temperature is not in the paper: logits are scaled as s = fl32(z * fl32(1/T))
    and the SCALED values are what is transmitted; the server's q_hat is the plain
    softmax of the received values;
  * "sample" = inverse CDF with a supplied uniform u in [0,1): first bucket whose
    cumulative sum exceeds u * total; dense distributions are scanned in ascending
    token index, sparse q_hat in canonical order (descending raw logit, ties by
    ascending index);
  * Algorithm 8's leaf branch samples from the target distribution of the leaf; the
    walk follows accepted children from the root.
"""
from __future__ import annotations

import numpy as np

STATUS_OK = 0
STATUS_NONFINITE = 1        # NaN or +inf among the logits of the row
STATUS_EMPTY = 2            # no finite logit / empty sparse set
STATUS_TOKEN_NOT_IN_SET = 4  # a draft token that is not in its sparse set


# ----------------------------------------------------------------------------------------------
# scaling and ordering
# ----------------------------------------------------------------------------------------------
def reciprocal_temperature(T) -> np.float32:
    """rT = fl32(1 / T) with T first rounded to fp32 (temperature is this build's reading; the
    paper has none)."""
    T32 = np.float32(T)
    if not (T32 > 0) or not np.isfinite(T32):
        raise ValueError("temperature must be a positive finite number")
    return np.float32(1.0 / np.float64(T32))


def scale(z, T) -> np.ndarray:
    """s_x = fl32(fl32(z_x) * rT): one IEEE fp32 multiplication per logit."""
    z32 = np.asarray(z, dtype=np.float32)
    return (z32 * reciprocal_temperature(T)).astype(np.float32)


def canonical_order(z) -> np.ndarray:
    """Tokens with a logit > -inf, ordered by raw logit descending, ties by ascending index
    (Section 3.1 sorts tokens in descending order of probability; the tie rule is this build's)."""
    z32 = np.asarray(z, dtype=np.float32)
    idx = np.arange(z32.shape[0])
    keep = idx[z32 > -np.inf]
    order = np.lexsort((keep, -z32[keep].astype(np.float64)))
    return keep[order]


def _row_status(z32) -> int:
    if np.isnan(z32).any() or (z32 == np.inf).any():
        return STATUS_NONFINITE
    if not (z32 > -np.inf).any():
        return STATUS_EMPTY
    return STATUS_OK


# ----------------------------------------------------------------------------------------------
# Section 3.1 / Solution 1: truncate one draft row
# ----------------------------------------------------------------------------------------------
def round_payload(s, payload: str) -> np.ndarray:
    """The scaled logits as they travel (Section 2.2: b_prob bits per value): "f32" unchanged, "f16" /
    "bf16" rounded to nearest-even to that 16-bit format and returned as the fp32 values the receiver decodes.
    Values beyond the format's finite range are clamped to it (a transmitted infinity would be useless)."""
    s = np.asarray(s, dtype=np.float32)
    if payload == "f32":
        return s.copy()
    if payload == "f16":
        return np.clip(s, -65504.0, 65504.0).astype(np.float16).astype(np.float32)
    if payload == "bf16":
        big = np.float32(3.3895313892515355e38)                  # largest finite bfloat16
        bits = np.clip(s, -big, big).view(np.uint32).astype(np.uint64)
        bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000  # round to nearest, ties to even
        return bits.astype(np.uint32).view(np.float32)
    raise ValueError(payload)


def truncate_row(z, T, top_k: int, top_p: float, k_cap: int, payload: str = "f32") -> dict:
    """Top-K / Top-rho truncation of one row of draft logits and renormalisation.

    Returns idx[count], logit[count] (fp32 scaled values, what is transmitted), prob[count]
    (q_hat, fp64), count, mass (rho = sum of q over the kept set; sigma = 1 - mass), margin_rho
    (relative distance of the nucleus test to its decision boundary, inf when the test did not
    decide the count) and status.  With a 16-bit payload the set is chosen as above, the emitted logits
    are round_payload of the kept ones, and q_hat is the softmax of those rounded values: it is what the
    receiver reconstructs, so it is what the sender must sample from.
    """
    z32 = np.asarray(z, dtype=np.float32)
    status = _row_status(z32)
    empty = dict(idx=np.zeros(0, np.int64), logit=np.zeros(0, np.float32), prob=np.zeros(0, np.float64),
                 count=0, mass=0.0, margin_rho=np.inf, status=status)
    if status != STATUS_OK:
        return empty
    s = scale(z32, T)
    order = canonical_order(z32)
    m = np.float64(s[order[0]])
    e = np.exp(s.astype(np.float64) - m)          # exp(-inf) = 0 for masked tokens
    Z = float(np.sum(e))
    k_sel = min(int(k_cap), order.shape[0])
    if top_k and top_k > 0:
        k_sel = min(k_sel, int(top_k))
    count = k_sel
    margin = np.inf
    if top_p is not None and 0.0 < float(np.float32(top_p)) < 1.0:
        C = np.cumsum(e[order])                   # descending-probability prefix masses
        thr = np.float64(np.float32(top_p)) * Z
        reach = np.nonzero(C >= thr)[0]
        m_rho = int(reach[0]) + 1 if reach.size else order.shape[0]
        if m_rho <= k_sel:
            count = m_rho
        # distance of the decision to flipping, for every boundary that could change `count`
        lo = min(m_rho, k_sel)
        cands = [abs(C[lo - 1] - thr)]
        if lo >= 2:
            cands.append(abs(C[lo - 2] - thr))
        margin = float(min(cands) / Z)
    head = order[:count]
    Csel = float(np.sum(e[head]))
    if payload == "f32":
        return dict(idx=head.astype(np.int64), logit=s[head].copy(), prob=e[head] / Csel, count=count,
                    mass=Csel / Z, margin_rho=margin, status=STATUS_OK)
    lg = round_payload(s[head], payload)
    return dict(idx=head.astype(np.int64), logit=lg, prob=sparse_probs(lg, count), count=count,
                mass=Csel / Z, margin_rho=margin, status=STATUS_OK)


def truncate(logits, T, top_k: int, top_p: float, k_cap: int, payload: str = "f32") -> dict:
    """truncate_row over [rows, V]; outputs padded to k_cap (idx -1, logit -inf, prob 0)."""
    logits = np.asarray(logits, dtype=np.float32)
    rows = logits.shape[0]
    out = dict(idx=np.full((rows, k_cap), -1, np.int32), logit=np.full((rows, k_cap), -np.inf, np.float32),
               prob=np.zeros((rows, k_cap), np.float64), count=np.zeros(rows, np.int32),
               mass=np.zeros(rows, np.float64), margin_rho=np.full(rows, np.inf),
               status=np.zeros(rows, np.int32))
    for r in range(rows):
        t = truncate_row(logits[r], T, top_k, top_p, k_cap, payload)
        c = t["count"]
        out["idx"][r, :c] = t["idx"]
        out["logit"][r, :c] = t["logit"]
        out["prob"][r, :c] = t["prob"]
        out["count"][r] = c
        out["mass"][r] = t["mass"]
        out["margin_rho"][r] = t["margin_rho"]
        out["status"][r] = t["status"]
    return out


# ----------------------------------------------------------------------------------------------
# sparse q_hat and sampling from it (Algorithm 2's sample step, Algorithm 4)
# ----------------------------------------------------------------------------------------------
def sparse_weights(logit, count: int) -> np.ndarray:
    """Unnormalised q_hat over a transmitted set: exp(s_i - s_0) in fp64 (s_0 is the largest: the
    set is in canonical order)."""
    s = np.asarray(logit[:count], dtype=np.float32).astype(np.float64)
    return np.exp(s - s[0]) if count > 0 else np.zeros(0)


def sparse_probs(logit, count: int) -> np.ndarray:
    """q_hat over a transmitted set = plain softmax of the received values."""
    w = sparse_weights(logit, count)
    return w / np.sum(w) if count > 0 else w


def inverse_cdf(weights, u):
    """First bucket whose cumulative weight exceeds u * total (sequential fp64 cumulative sum).
    Returns (bucket, margin) with margin = relative distance of u*total to the nearest edge of the
    chosen bucket; bucket -1 when the total is not positive."""
    w = np.asarray(weights, dtype=np.float64)
    c = np.cumsum(w)
    total = c[-1] if c.size else 0.0
    if not (total > 0.0):
        return -1, np.inf
    t = np.float64(np.float32(u)) * total
    y = int(np.searchsorted(c, t, side="right"))
    if y >= w.shape[0]:                      # cannot happen for u < 1; keep the scan total
        y = int(np.nonzero(w > 0)[0][-1])
    below = c[y - 1] if y > 0 else 0.0
    margin = min(abs(c[y] - t), abs(t - below)) / total
    return y, float(margin)


def sample_row(logit, count: int, u, without_replacement: bool = False):
    """Draw len(u) slots from q_hat (Algorithm 4 draws the k candidates i.i.d.; the
    without-replacement variant removes each drawn slot and renormalises over the rest).
    Returns (slots int array, margins)."""
    u = np.atleast_1d(np.asarray(u, dtype=np.float32))
    slots = np.full(u.shape[0], -1, np.int32)
    margins = np.full(u.shape[0], np.inf)
    if count <= 0:
        return slots, margins
    w = sparse_weights(logit, count).copy()
    for c in range(u.shape[0]):
        y, mg = inverse_cdf(w, u[c])
        slots[c], margins[c] = y, mg
        if without_replacement and y >= 0:
            w[y] = 0.0
    return slots, margins


def sample(idx, logit, count, u, without_replacement: bool = False):
    """sample_row over rows: idx/logit [rows, k_cap], count [rows], u [rows, n]."""
    idx = np.asarray(idx)
    rows = idx.shape[0]
    u = np.asarray(u, dtype=np.float32).reshape(rows, -1)
    n = u.shape[1]
    token = np.full((rows, n), -1, np.int32)
    slot = np.full((rows, n), -1, np.int32)
    margin = np.full((rows, n), np.inf)
    for r in range(rows):
        s, mg = sample_row(logit[r], int(count[r]), u[r], without_replacement)
        slot[r] = s
        margin[r] = mg
        ok = s >= 0
        token[r, ok] = idx[r, s[ok]]
    return dict(token=token, slot=slot, margin=margin)


# ----------------------------------------------------------------------------------------------
# dense target distribution
# ----------------------------------------------------------------------------------------------
def dense_probs(t, T) -> np.ndarray:
    """p = softmax(scale(t, T)) in fp64."""
    s = scale(t, T).astype(np.float64)
    m = np.max(s)
    e = np.exp(s - m)
    return e / np.sum(e)


def scatter_sparse(V: int, q_idx, q_prob) -> np.ndarray:
    """Dense length-V vector holding q_hat on its set and 0 elsewhere."""
    q = np.zeros(V, np.float64)
    q[np.asarray(q_idx, dtype=np.int64)] = q_prob
    return q


# ----------------------------------------------------------------------------------------------
# Algorithm 3: single-candidate verification of one sequence
# ----------------------------------------------------------------------------------------------
def verify_chain_seq(target, T, q_idx, q_logit, q_count, tokens, u_accept, u_resample) -> dict:
    """target [gamma+1, V]; q_idx/q_logit [gamma, k_cap]; q_count, tokens, u_accept [gamma];
    u_resample [gamma+1].  Walks j = 1..gamma: accept x_j iff u_j < min(1, p_j(x_j)/q_hat_j(x_j));
    on the first rejection resample from norm(max(0, p_j - q_hat_j)) and stop; if everything is
    accepted draw the bonus token from p_{gamma+1}."""
    target = np.asarray(target, dtype=np.float32)
    gamma = target.shape[0] - 1
    V = target.shape[1]
    out_tokens = np.full(gamma + 1, -1, np.int32)
    ratio = np.full(gamma, np.nan)
    beta_hat = np.full(gamma, np.nan)
    acc_margin = np.full(gamma, np.inf)
    status = 0
    res = dict(accept_len=0, tokens=out_tokens, ratio=ratio, beta_hat=beta_hat, accept_margin=acc_margin,
               cdf_margin=np.inf, status=0)
    for j in range(gamma):
        st = _row_status(target[j])
        if st != STATUS_OK:
            res["status"] = status | st
            res["accept_len"] = j
            return res                      # no token can be produced from a broken row
        p = dense_probs(target[j], T)
        cnt = int(q_count[j])
        qh = sparse_probs(q_logit[j], cnt)
        ids = np.asarray(q_idx[j][:cnt], dtype=np.int64)
        q_dense = scatter_sparse(V, ids, qh)
        beta_hat[j] = float(np.sum(np.minimum(p[ids], qh)))
        x = int(tokens[j])
        where = np.nonzero(ids == x)[0]
        accepted = False
        if where.size == 0:
            status |= STATUS_TOKEN_NOT_IN_SET
            ratio[j] = -1.0
        else:
            ratio[j] = p[x] / qh[where[0]]
            bound = min(1.0, ratio[j])
            uj = np.float64(np.float32(u_accept[j]))
            accepted = bool(uj < bound)
            acc_margin[j] = abs(uj - bound)
        if accepted:
            out_tokens[j] = x
            continue
        r = np.maximum(0.0, p - q_dense)
        y, mg = inverse_cdf(r, u_resample[j])
        if y < 0:                           # defensive: an all-zero residual, fall back to p
            y, mg = inverse_cdf(p, u_resample[j])
        out_tokens[j] = y
        res.update(accept_len=j, cdf_margin=mg, status=status)
        return res
    st = _row_status(target[gamma])
    if st != STATUS_OK:
        res.update(accept_len=gamma, status=status | st)
        return res
    y, mg = inverse_cdf(dense_probs(target[gamma], T), u_resample[gamma])
    out_tokens[gamma] = y
    res.update(accept_len=gamma, cdf_margin=mg, status=status)
    return res


def verify_chain(target, T, q_idx, q_logit, q_count, tokens, u_accept, u_resample) -> dict:
    """verify_chain_seq over a batch: target [B, gamma+1, V], sparse sets [B, gamma, k_cap]."""
    target = np.asarray(target)
    B, g1, _ = target.shape
    gamma = g1 - 1
    out = dict(accept_len=np.zeros(B, np.int32), tokens=np.full((B, g1), -1, np.int32),
               ratio=np.full((B, gamma), np.nan), beta_hat=np.full((B, gamma), np.nan),
               accept_margin=np.full((B, gamma), np.inf), cdf_margin=np.full(B, np.inf),
               status=np.zeros(B, np.int32))
    for b in range(B):
        r = verify_chain_seq(target[b], T, q_idx[b], q_logit[b], q_count[b], tokens[b], u_accept[b],
                             u_resample[b])
        for k in ("accept_len", "cdf_margin", "status"):
            out[k][b] = r[k]
        for k in ("tokens", "ratio", "beta_hat", "accept_margin"):
            out[k][b] = r[k]
    return out


# ----------------------------------------------------------------------------------------------
# Algorithm 5: multi-candidate verification at one node
# ----------------------------------------------------------------------------------------------
def mcveri(p, q_idx, q_prob, cands, u_accept, u_resample, without_replacement: bool = False) -> dict:
    """p: dense fp64 target distribution of the node; (q_idx, q_prob): sparse q_hat; cands[k]
    candidate tokens (-1 = absent); u_accept[k]; u_resample scalar.
    P^(1) = P; candidate i is accepted iff u_i < min(1, p^(i)(x_i)/q^(i)(x_i)); otherwise
    p^(i+1) = norm(max(0, p^(i) - q^(i))); after k rejections the output is a sample of P^(k+1).

    without_replacement = False is Algorithm 5 as printed: q^(i) = q_hat at every step, exact when the
    candidates are i.i.d. draws from q_hat (Algorithm 4).
    without_replacement = True is the rule for candidates drawn one after the other from q_hat without
    replacement (the direction Section 4.2 only cites): candidate i was drawn from q^(i) = q_hat with
    x_1..x_{i-1} removed and the rest renormalised, so stage i is single-candidate speculative sampling
    with target p^(i) and THAT proposal, which keeps the output distributed as P.

    Returns token, slot (accepted candidate number or -1), ratios, accept margins, the cdf margin, the
    stage acceptance rates beta^(i) = sum_x min(q^(i), p^(i)) met on the way, and per candidate the factor
    prod_{j<i} 1/Z_j by which an error in p is magnified in p^(i) (Z_j = sum_x max(0, p^(j) - q^(j)) <= 1 is
    the normaliser of update j)."""
    p_i = np.asarray(p, dtype=np.float64).copy()
    V = p_i.shape[0]
    ids = np.asarray(q_idx, dtype=np.int64)
    q_hat = scatter_sparse(V, ids, q_prob)
    q_i = q_hat.copy()                      # proposal of the current stage
    k = len(cands)
    ratio = np.full(k, np.nan)
    margin = np.full(k, np.inf)
    amp = np.ones(k)
    gain = 1.0
    betas = []
    beta = np.full(k, np.nan)               # the same rates, by candidate number
    status = 0
    for i in range(k):
        x = int(cands[i])
        if x < 0:
            continue
        amp[i] = gain
        betas.append(float(np.sum(np.minimum(q_i, p_i))))
        beta[i] = betas[-1]
        if q_i[x] <= 0.0:                   # not in the set (or, without replacement, drawn before)
            status |= STATUS_TOKEN_NOT_IN_SET
            ratio[i] = -1.0
            accepted = False
        else:
            ratio[i] = p_i[x] / q_i[x]
            bound = min(1.0, ratio[i])
            ui = np.float64(np.float32(u_accept[i]))
            accepted = bool(ui < bound)
            margin[i] = abs(ui - bound)
        if accepted:
            return dict(token=x, slot=i, ratio=ratio, accept_margin=margin, cdf_margin=np.inf,
                        betas=betas, beta=beta, status=status, amp=amp)
        r = np.maximum(0.0, p_i - q_i)
        Zr = np.sum(r)
        if Zr > 0.0:                        # always true after a rejection in exact arithmetic
            p_i = r / Zr
            gain /= Zr
        if without_replacement and q_hat[x] > 0.0:
            q_hat[x] = 0.0                  # x leaves the urn; the next candidate came from what is left
            rest = np.sum(q_hat)
            q_i = q_hat / rest if rest > 0.0 else q_hat.copy()
    y, mg = inverse_cdf(p_i, u_resample)
    return dict(token=y, slot=-1, ratio=ratio, accept_margin=margin, cdf_margin=mg, betas=betas, beta=beta,
                status=status, amp=amp)


# ----------------------------------------------------------------------------------------------
# Section 4.1 tree layout and Algorithm 8
# ----------------------------------------------------------------------------------------------
def tree_layout(expansion) -> dict:
    """Breadth-first layout of an expansion-configured token tree: layer widths
    W_l = prod_{j<=l} k_j, layer offsets, node counts; |Q| = number of non-leaf nodes
    = 1 + sum_{l=1}^{L-1} prod_{i<=l} k_i."""
    widths = [1]
    for kk in expansion:
        widths.append(widths[-1] * int(kk))
    offsets = np.concatenate([[0], np.cumsum(widths)]).astype(np.int64)
    return dict(depth=len(expansion), widths=widths, offsets=offsets, n_nodes=int(offsets[-1]),
                n_internal=int(offsets[-2]))


def child_node(layout, expansion, node: int, slot: int) -> int:
    """Node id of the slot-th child (0-based) of `node`: the i-th node of layer l (0-based i) owns
    nodes i*k_{l+1} .. (i+1)*k_{l+1}-1 of layer l+1."""
    off = layout["offsets"]
    layer = int(np.searchsorted(off, node, side="right")) - 1
    i = node - int(off[layer])
    return int(off[layer + 1]) + i * int(expansion[layer]) + slot


def verify_tree_seq(target, T, expansion, q_idx, q_logit, q_count, cand_tokens, u_accept,
                    u_resample, without_replacement: bool = False) -> dict:
    """target [N_nodes, V]; sparse sets [N_int, k_cap]; cand_tokens, u_accept [N_nodes-1] (entry
    n-1 belongs to node n); u_resample [N_nodes].  Runs Algorithm 5 at every non-leaf node, draws a
    target sample at every leaf, then walks from the root through accepted children."""
    target = np.asarray(target, dtype=np.float32)
    lay = tree_layout(expansion)
    n_nodes, n_int, depth = lay["n_nodes"], lay["n_internal"], lay["depth"]
    node_token = np.full(n_nodes, -1, np.int32)
    node_slot = np.full(n_nodes, -1, np.int32)
    ratio = np.full(max(n_nodes - 1, 0), np.nan)
    beta = np.full(max(n_nodes - 1, 0), np.nan)
    acc_margin = np.full(max(n_nodes - 1, 0), np.inf)
    amp = np.ones(max(n_nodes - 1, 0))
    cdf_margin = np.full(n_nodes, np.inf)
    status = 0
    for n in range(n_nodes):
        st = _row_status(target[n])
        if st != STATUS_OK:
            status |= st
            continue
        p = dense_probs(target[n], T)
        if n < n_int:
            layer = int(np.searchsorted(lay["offsets"], n, side="right")) - 1
            k = int(expansion[layer])
            c0 = child_node(lay, expansion, n, 0)
            cnt = int(q_count[n])
            qh = sparse_probs(q_logit[n], cnt)
            r = mcveri(p, q_idx[n][:cnt], qh, cand_tokens[c0 - 1:c0 - 1 + k], u_accept[c0 - 1:c0 - 1 + k],
                       u_resample[n], without_replacement)
            node_token[n], node_slot[n] = r["token"], r["slot"]
            ratio[c0 - 1:c0 - 1 + k] = r["ratio"]
            beta[c0 - 1:c0 - 1 + k] = r["beta"]
            acc_margin[c0 - 1:c0 - 1 + k] = r["accept_margin"]
            amp[c0 - 1:c0 - 1 + k] = r["amp"]
            cdf_margin[n] = r["cdf_margin"]
            status |= r["status"]
        else:
            y, mg = inverse_cdf(p, u_resample[n])
            node_token[n], cdf_margin[n] = y, mg
    seq = np.full(depth + 1, -1, np.int32)
    path = []
    n, length = 0, 0
    while True:
        path.append(n)
        seq[length] = node_token[n]
        length += 1
        if n < n_int and node_slot[n] >= 0:
            n = child_node(lay, expansion, n, int(node_slot[n]))
        else:
            break
    return dict(node_token=node_token, node_slot=node_slot, seq=seq, len=length, path=path, ratio=ratio, beta=beta,
                accept_margin=acc_margin, amp=amp, cdf_margin=cdf_margin, status=status)


def verify_tree(target, T, expansion, q_idx, q_logit, q_count, cand_tokens, u_accept, u_resample,
                without_replacement: bool = False) -> dict:
    """verify_tree_seq over a batch (leading dimension B on every array)."""
    target = np.asarray(target)
    B = target.shape[0]
    lay = tree_layout(expansion)
    out = dict(node_token=np.full((B, lay["n_nodes"]), -1, np.int32),
               node_slot=np.full((B, lay["n_nodes"]), -1, np.int32),
               seq=np.full((B, lay["depth"] + 1), -1, np.int32), len=np.zeros(B, np.int32),
               ratio=np.full((B, lay["n_nodes"] - 1), np.nan), beta=np.full((B, lay["n_nodes"] - 1), np.nan),
               accept_margin=np.full((B, lay["n_nodes"] - 1), np.inf), amp=np.ones((B, lay["n_nodes"] - 1)),
               cdf_margin=np.full((B, lay["n_nodes"]), np.inf), status=np.zeros(B, np.int32), path=[])
    for b in range(B):
        r = verify_tree_seq(target[b], T, expansion, q_idx[b], q_logit[b], q_count[b], cand_tokens[b],
                            u_accept[b], u_resample[b], without_replacement)
        for k in ("node_token", "node_slot", "seq", "ratio", "beta", "accept_margin", "amp", "cdf_margin"):
            out[k][b] = r[k]
        out["len"][b] = r["len"]
        out["status"][b] = r["status"]
        out["path"].append(r["path"])
    return out


# ----------------------------------------------------------------------------------------------
# Section 3.2: what truncation to the first K entries does to the acceptance rate
# ----------------------------------------------------------------------------------------------
def truncation_stats_row(target_row, T, idx, logit, count, k_list) -> dict:
    """One target row against the nested prefixes of one truncated set.  The set is in canonical order, so
    its first K entries are the Top-K set of the same draft distribution.  For every K of k_list:
      keep[K] = sum_{i<K} q_hat_i, the share of the whole set's mass that the prefix holds (q_hat = softmax of
                the received values over the whole set);
      beta[K] = sum_x min(q_hat_K(x), p(x)) with q_hat_K the prefix renormalised (the acceptance rate under
                truncation, Section 3.2; 1 - TV(q_hat_K, p) by Lemma 1).
    K larger than the set's size means the whole set.  A broken row gives NaN."""
    target_row = np.asarray(target_row, dtype=np.float32)
    ks = [int(k) for k in k_list]
    keep = np.full(len(ks), np.nan)
    beta = np.full(len(ks), np.nan)
    st = _row_status(target_row)
    cnt = int(count)
    if st != STATUS_OK or cnt <= 0:
        return dict(keep=keep, beta=beta, status=st if st != STATUS_OK else STATUS_EMPTY)
    p = dense_probs(target_row, T)
    qh = sparse_probs(logit, cnt)
    ids = np.asarray(idx[:cnt], dtype=np.int64)
    for j, K in enumerate(ks):
        k = min(max(K, 1), cnt)
        c = float(np.sum(qh[:k]))
        keep[j] = c
        beta[j] = float(np.sum(np.minimum(qh[:k] / c, p[ids[:k]])))
    return dict(keep=keep, beta=beta, status=STATUS_OK)


def truncation_stats(target_rows, T, idx, logit, count, k_list) -> dict:
    """truncation_stats_row over rows: target_rows [n, V], sets [n, k_cap]."""
    target_rows = np.asarray(target_rows, dtype=np.float32)
    n = target_rows.shape[0]
    out = dict(keep=np.full((n, len(k_list)), np.nan), beta=np.full((n, len(k_list)), np.nan), status=np.zeros(n, np.int32))
    for r in range(n):
        one = truncation_stats_row(target_rows[r], T, idx[r], logit[r], count[r], k_list)
        out["keep"][r], out["beta"][r], out["status"][r] = one["keep"], one["beta"], one["status"]
    return out


# ----------------------------------------------------------------------------------------------
# Section 4.3: acceptance rates of the k candidates of multi-candidate verification
# ----------------------------------------------------------------------------------------------
def multi_candidate_rates(p, q_idx, q_prob, k: int) -> dict:
    """beta^(j), j = 1..k, and the total acceptance rate theta of Section 4.3 for one node, under Algorithm 5
    as printed (candidates i.i.d. from q_hat, the same q_hat at every stage).  P^(1) = P and
    p^(j+1) = norm(max(0, p^(j) - q_hat)) do not depend on which tokens were drawn, so the rates are functions
    of (p, q_hat) alone:
      beta^(j) = sum_x min(q_hat(x), p^(j)(x))                       (the lemma of Section 4.3)
      theta    = beta^(1) + sum_{i=2..k} beta^(i) prod_{j<i} (1 - beta^(j)).
    A stage whose residual is empty (beta^(j) = 1: the candidate is always accepted) ends the recursion; the
    rates of the stages after it, which are never reached, are NaN and add nothing to theta."""
    p_j = np.asarray(p, dtype=np.float64).copy()
    q_hat = scatter_sparse(p_j.shape[0], np.asarray(q_idx, dtype=np.int64), q_prob)
    beta = np.full(int(k), np.nan)
    theta = 0.0
    reach = 1.0                                  # probability that stage j is reached: prod_{i<j} (1 - beta^(i))
    for j in range(int(k)):
        beta[j] = float(np.sum(np.minimum(q_hat, p_j)))
        theta += beta[j] * reach
        reach *= 1.0 - beta[j]
        r = np.maximum(0.0, p_j - q_hat)
        Zr = float(np.sum(r))
        if not (Zr > 0.0):
            break
        p_j = r / Zr
    return dict(beta=beta, theta=theta)


def multi_candidate_stats(target_rows, T, idx, logit, count, k: int) -> dict:
    """multi_candidate_rates over rows: target_rows [n, V] against truncated sets [n, k_cap] (p = softmax of the
    scaled target row, q_hat = softmax of the received values).  A broken row or an empty set gives NaN."""
    target_rows = np.asarray(target_rows, dtype=np.float32)
    n = target_rows.shape[0]
    out = dict(beta=np.full((n, int(k)), np.nan), theta=np.full(n, np.nan), status=np.zeros(n, np.int32))
    for r in range(n):
        st = _row_status(target_rows[r])
        cnt = int(count[r])
        if st != STATUS_OK or cnt <= 0:
            out["status"][r] = st if st != STATUS_OK else STATUS_EMPTY
            continue
        one = multi_candidate_rates(dense_probs(target_rows[r], T), np.asarray(idx[r][:cnt]), sparse_probs(logit[r], cnt), k)
        out["beta"][r], out["theta"][r] = one["beta"], one["theta"]
    return out


# ----------------------------------------------------------------------------------------------
# Section 2.2: payload model, and the wire format of a batch of truncated sets
# ----------------------------------------------------------------------------------------------
def index_bits(V: int) -> int:
    """b_idx = ceil(log2 |V|)."""
    return int(np.ceil(np.log2(V)))


def payload_bits(n_entries: int, b_prob: int, b_idx: int) -> int:
    """D = n * (b_prob + b_idx): n = |V| for a dense distribution, n = K for a truncated one."""
    return int(n_entries) * (int(b_prob) + int(b_idx))


def _value_bits16(logit, payload: str) -> np.ndarray:
    """The 16-bit pattern of every (already rounded) value."""
    v = round_payload(logit, payload)
    if payload == "f16":
        return v.astype(np.float16).view(np.uint16).astype(np.uint64)
    if payload == "bf16":
        return (v.view(np.uint32) >> 16).astype(np.uint64)
    raise ValueError(payload)


def pack_rows(idx, logit, count, V: int, payload: str) -> dict:
    """Wire format of truncated sets (the paper fixes only the size, Section 2.2: K pairs of a b_idx-bit
    token id and a b_prob-bit value; the layout is this build's).  The stream of one row, least significant
    bit first: 16 bits count, then per kept entry, in canonical order, b_idx = ceil(log2 V) bits of token id
    followed by the 16 bits of the value (binary16 or bfloat16).  Rows are padded with zero bits to whole
    32-bit words and concatenated; row_offset[r] is the first word of row r, row_offset[rows] the total.
    Bit p of a row's stream is bit p % 32 of its word p // 32.  payload_bits counts only the pairs:
    sum_r count_r * (b_idx + 16), the D of Section 2.2."""
    idx = np.asarray(idx)
    count = np.asarray(count, dtype=np.int64)
    rows = idx.shape[0]
    b_idx = index_bits(V)
    E = b_idx + 16
    n_words = (16 + count * E + 31) // 32
    row_offset = np.concatenate([[0], np.cumsum(n_words)]).astype(np.int64)
    words = np.zeros(int(row_offset[-1]), np.uint32)
    for r in range(rows):
        c = int(count[r])
        stream = int(c)                                     # a Python integer as the bit stream
        vals = _value_bits16(np.asarray(logit[r][:c], dtype=np.float32), payload)
        for i in range(c):
            entry = int(idx[r][i]) | (int(vals[i]) << b_idx)
            stream |= entry << (16 + i * E)
        for wd in range(int(n_words[r])):
            words[row_offset[r] + wd] = (stream >> (32 * wd)) & 0xFFFFFFFF
    return dict(words=words, row_offset=row_offset, payload_bits=int(np.sum(count)) * E, b_idx=b_idx)


def unpack_rows(words, row_offset, rows: int, k_cap: int, V: int, payload: str) -> dict:
    """Inverse of pack_rows: idx [rows, k_cap] (-1 beyond count), logit (fp32 of the received values, -inf
    beyond count), count."""
    words = np.asarray(words, dtype=np.uint32)
    b_idx = index_bits(V)
    E = b_idx + 16
    out = dict(idx=np.full((rows, k_cap), -1, np.int32), logit=np.full((rows, k_cap), -np.inf, np.float32),
               count=np.zeros(rows, np.int32))
    for r in range(rows):
        seg = words[int(row_offset[r]):int(row_offset[r + 1])]
        stream = 0
        for wd, x in enumerate(seg):
            stream |= int(x) << (32 * wd)
        c = stream & 0xFFFF
        out["count"][r] = c
        for i in range(min(c, k_cap)):
            entry = (stream >> (16 + i * E)) & ((1 << E) - 1)
            out["idx"][r, i] = entry & ((1 << b_idx) - 1)
            bits = np.array([entry >> b_idx], dtype=np.uint16)
            if payload == "f16":
                out["logit"][r, i] = bits.view(np.float16).astype(np.float32)[0]
            else:
                out["logit"][r, i] = (bits.astype(np.uint32) << 16).view(np.float32)[0]
    return out
