"""CPU oracle for the budgeted MoE-layer forward of MoE-Spec.  TEST INFRASTRUCTURE.

A plain, slow, fp64 numpy implementation of what the hot path computes, written
step by step from the paper's definitions so that it can be checked against the
paper by eye.  It shares no code with the HIP path and is never used by it:
only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this module.

Notation follows the paper: ``M`` draft-tree tokens ``h_t`` of size ``d``,
``N`` experts, per-token top-``k``, budget ``B``, shortlist ``S``.

Steps and the passages they follow
  router_logits / routing_probs   Eq. (1): softmax of the router projection
  top_k / mixing_weights          Section 2.1: T_k(h) and the mixing weights g-bar
  aggregate_scores                Eq. (5), Algorithm 1 stage 2: s_i = sum_t g_i(h_t)
  shortlist                       Section 3.2 "Router-Based Ranking": B highest s_i
  restrict_truncation             Eq. (7) and the paragraph after it
  restrict_substitution           Eq. (8) and the paragraph after it
  expert_union                    Eq. (3)
  expert                          SwiGLU feed-forward (the paper leaves E_i open;
                                  the workloads fix SwiGLU without biases)
  combine / layer_forward         Eq. (2), (7), (8); Algorithm 1
  calibration_counts / static_shortlist
                                  Eq. (4), "Static Ranking": selection frequency over
                                  calibration tokens and the B most frequent experts
  coverage_curve                  cumulative routing probability captured by the top-B
                                  experts, B = 1..N (Section 4.6)
  oracle_ranking                  Eq. (6), "Oracle Ranking": greedy selection that minimises the
                                  reconstruction error against the gold output O*
  reconstruction_error            Section 4.5: ||O_S - O*||^2 / ||O*||^2, O* from Eq. (2)
  rms_scale / layer_stack         the stack of layers joined by the residual stream (the layer-stack workload),
                                  with the optional unit-RMS scaling of each layer's input
  segments                        the per-expert grouping of surviving
                                  (token, slot) pairs; defined here, the paper's
                                  batched matmul (Appendix C) hides it

Readings where the paper is silent
  * ties in every ranking go to the lowest expert id;
  * rankings compare the routing probabilities g (as the paper words it), in fp64;
  * a router bias ``b`` is added to the projection when given (the workloads use
    one to make routing heavy-tailed); ``b=None`` is Eq. (1) as printed;
  * sigmoid-gated routing (named by the paper as an open case) replaces only the gate: g_i = sigmoid of the
    logit, and T_k, Eq. (5), Eq. (7)/(8) are applied to those scores unchanged;
  * substitution weights are the full-softmax g_i restricted to the new set,
    renormalised over that set when the architecture renormalises;
  * Eq. (6) writes the partial sum over all j in S + {i} with raw g; it is read as the sum over
    (S + {i}) intersected with T_k(h_t) with the mixing weights of Eq. (2), so that the full set
    reproduces the gold output O* exactly (an expert outside a token's top-k contributes nothing).

Every function is pinned by tests/test_oracle_*.py against closed forms,
brute force on tiny inputs, invariants the paper states and library routines.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

TRUNCATE = 0
SUBSTITUTE = 1


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


# --------------------------------------------------------------------------- Eq. (1)
def router_logits(h, w_router, b_router=None) -> np.ndarray:
    """logit[t, i] = w_i . h_t (+ b_i).  h[M, d], w_router[N, d] -> [M, N] fp64."""
    h, w_router = _f64(h), _f64(w_router)
    logits = np.empty((h.shape[0], w_router.shape[0]), dtype=np.float64)
    for t in range(h.shape[0]):
        for i in range(w_router.shape[0]):
            logits[t, i] = np.dot(w_router[i], h[t])      # one routine for every (t, i): equal rows give equal logits
            if b_router is not None:
                logits[t, i] += float(b_router[i])
    return logits


SOFTMAX, SIGMOID = "softmax", "sigmoid"


def routing_probs(logits, gate: str = SOFTMAX) -> np.ndarray:
    """g[t, :] = softmax over all N experts of logit[t, :] (max-subtracted), Eq. (1).

    gate="sigmoid": g[t, i] = 1 / (1 + exp(-logit[t, i])), every expert gated on its own (the routing scheme the
    paper's limitations section names as an open case; everything downstream - T_k, Eq. (5), Eq. (7)/(8) - is
    applied to these scores unchanged)."""
    logits = _f64(logits)
    g = np.empty_like(logits)
    for t in range(logits.shape[0]):
        if gate == SIGMOID:
            g[t] = 1.0 / (1.0 + np.exp(-logits[t]))
        elif gate == SOFTMAX:
            e = np.exp(logits[t] - np.max(logits[t]))
            g[t] = e / np.sum(e)
        else:
            raise ValueError("unknown gate")
    return g


# --------------------------------------------------------------------------- Section 2.1
def rank_desc(values: Sequence[float], candidates: Optional[Sequence[int]] = None) -> List[int]:
    """Candidate indices ordered by (value descending, index ascending)."""
    idx = range(len(values)) if candidates is None else candidates
    return sorted(idx, key=lambda i: (-float(values[i]), int(i)))


def top_k(g_row, k: int) -> List[int]:
    """T_k(h): the k experts with the largest routing probability, best first."""
    return rank_desc(g_row)[:k]


def mixing_weights(g_row, ids: Sequence[int], renorm: bool) -> List[float]:
    """g-bar over the selected set: raw g_i, or g_i / sum_{j in ids} g_j.

    If every selected expert has probability exactly 0 in fp64 (router logits more than 745 apart: substitution
    inside a shortlist that holds none of the token's own experts) the renormalised weights are 0/0; the paper
    does not cover the case and the reading is IEEE arithmetic: NaN for every slot of that token."""
    if renorm:
        denom = 0.0
        for j in ids:
            denom += float(g_row[j])
        if denom == 0.0:
            return [float("nan")] * len(ids)
        return [float(g_row[i]) / denom for i in ids]
    return [float(g_row[i]) for i in ids]


def route(h, w_router, b_router, k: int, renorm: bool, gate: str = SOFTMAX):
    """Unbudgeted routing of every token: (g[M,N], ids[M,k], w[M,k])."""
    g = routing_probs(router_logits(h, w_router, b_router), gate)
    M = g.shape[0]
    ids = np.zeros((M, k), dtype=np.int32)
    w = np.zeros((M, k), dtype=np.float64)
    for t in range(M):
        sel = top_k(g[t], k)
        ids[t] = sel
        w[t] = mixing_weights(g[t], sel, renorm)
    return g, ids, w


# --------------------------------------------------------------------------- Eq. (3)
def expert_union(topk_ids) -> List[int]:
    """E(D): union over tokens of the natural top-k sets, ascending ids."""
    return sorted({int(i) for i in np.asarray(topk_ids).ravel()})


# --------------------------------------------------------------------------- Eq. (5)
def aggregate_scores(g) -> np.ndarray:
    """s_i = sum over the M tree tokens of g_i(h_t), over all N experts."""
    g = _f64(g)
    s = np.zeros(g.shape[1], dtype=np.float64)
    for t in range(g.shape[0]):
        s = s + g[t]
    return s


def shortlist(scores, B: int) -> List[int]:
    """S: the B experts with the highest aggregate score, best first."""
    return rank_desc(scores)[:B]


def coverage(scores, S: Sequence[int]) -> float:
    """Fraction of the tree's routing mass held by the shortlist."""
    s = _f64(scores)
    return float(sum(s[i] for i in S) / np.sum(s))


def coverage_curve(scores) -> np.ndarray:
    """curve[B-1] = share of the tree's routing probability held by the B highest-scoring experts,
    B = 1..N (Section 4.6: cumulative routing probability captured by the top-B experts)."""
    s = _f64(scores)
    total = 0.0
    for i in range(s.shape[0]):
        total = total + s[i]
    curve = np.zeros(s.shape[0], dtype=np.float64)
    acc = 0.0
    for r, i in enumerate(rank_desc(s)):
        acc = acc + s[i]
        curve[r] = acc / total
    return curve


# --------------------------------------------------------------------------- Eq. (4)
def calibration_counts(topk_ids, n_experts: int, counts=None) -> np.ndarray:
    """c_i = number of calibration tokens h with i in T_k(h); `counts` (int64) carries earlier batches."""
    c = np.zeros(n_experts, dtype=np.int64) if counts is None else np.array(counts, dtype=np.int64)
    for row in np.asarray(topk_ids):
        for i in row:
            if i >= 0:
                c[int(i)] += 1
    return c


def static_shortlist(counts, B: int) -> List[int]:
    """The B experts with the highest selection frequency, most frequent first (ties: lowest id)."""
    c = [int(v) for v in counts]
    return sorted(range(len(c)), key=lambda i: (-c[i], i))[:B]


# --------------------------------------------------------------------------- Eq. (6)
def expert_contributions(h, topk_ids, topk_w, w_gate, w_up, w_down, n_experts: int) -> np.ndarray:
    """C[i, t, :] = g-bar_i(h_t) * E_i(h_t) if i is in T_k(h_t), else 0; the gold output is O* = sum_i C[i]."""
    h = _f64(h)
    bank = _ExpertBank(w_gate, w_up, w_down)
    C = np.zeros((n_experts, h.shape[0], h.shape[1]), dtype=np.float64)
    for t in range(h.shape[0]):
        for j in range(np.asarray(topk_ids).shape[1]):
            i = int(topk_ids[t][j])
            if i >= 0:
                C[i, t] = float(topk_w[t][j]) * expert(h[t], *bank.get(i))
    return C


def oracle_ranking(C, B: int):
    """Greedy oracle of Eq. (6) on the per-expert contributions C[N, M, d].

    Starting from the empty set, B times add the expert i outside S that minimises
    sum_t ||O*_t - sum_{j in S + {i}} C[j, t]||^2 (ties: lowest id).  Returns the experts in the order
    they were added and, after each addition, that error divided by ||O*||^2.
    """
    C = _f64(C)
    N = C.shape[0]
    gold = np.zeros(C.shape[1:], dtype=np.float64)
    for i in range(N):
        gold = gold + C[i]
    denom = float(np.sum(gold * gold))
    partial = np.zeros_like(gold)
    S: List[int] = []
    errs: List[float] = []
    for _ in range(B):
        best, best_err = -1, 0.0
        for i in range(N):
            if i in S:
                continue
            r = gold - (partial + C[i])
            e = float(np.sum(r * r))
            if best < 0 or e < best_err:
                best, best_err = i, e
        S.append(best)
        partial = partial + C[best]
        errs.append(best_err / denom)
    return S, np.asarray(errs, dtype=np.float64)


# --------------------------------------------------------------------------- Section 4.5
def reconstruction_error(out_budgeted, out_full) -> float:
    """||O_S - O*||^2 / ||O*||^2 over all tokens of the layer (squared Frobenius norms)."""
    a, b = _f64(out_budgeted), _f64(out_full)
    num = den = 0.0
    for t in range(a.shape[0]):
        diff = a[t] - b[t]
        num = num + float(np.dot(diff, diff))
        den = den + float(np.dot(b[t], b[t]))
    return num / den


# --------------------------------------------------------------------------- Eq. (7)
def restrict_truncation(topk_ids, topk_w, S: Sequence[int]):
    """Keep each token's natural top-k slots that fall inside S, weights unchanged.

    Dropped slots get id -1 and weight 0; slot order is kept.
    """
    topk_ids = np.asarray(topk_ids)
    in_S = set(int(i) for i in S)
    ids = np.full(topk_ids.shape, -1, dtype=np.int32)
    w = np.zeros(topk_ids.shape, dtype=np.float64)
    for t in range(topk_ids.shape[0]):
        for j in range(topk_ids.shape[1]):
            if int(topk_ids[t, j]) in in_S:
                ids[t, j] = topk_ids[t, j]
                w[t, j] = topk_w[t][j]
    return ids, w


# --------------------------------------------------------------------------- Eq. (8)
def restrict_substitution(g, S: Sequence[int], k: int, renorm: bool):
    """Top-k within S by g_i(h_t) for every token; every token gets exactly k experts."""
    if len(S) < k:
        raise ValueError("substitution needs a shortlist of at least k experts")
    g = _f64(g)
    M = g.shape[0]
    ids = np.zeros((M, k), dtype=np.int32)
    w = np.zeros((M, k), dtype=np.float64)
    for t in range(M):
        sel = rank_desc(g[t], candidates=list(S))[:k]
        ids[t] = sel
        w[t] = mixing_weights(g[t], sel, renorm)
    return ids, w


# --------------------------------------------------------------------------- grouping
def segments(tok_ids, S: Sequence[int]):
    """Group surviving (token, slot) pairs by expert.

    Returns ``seg_expert`` (S in ascending id), ``seg_off`` (len(S)+1 offsets) and
    ``perm`` (flat pair index ``t*k + slot`` of each position), pairs ordered by
    (expert id ascending, token ascending).
    """
    tok_ids = np.asarray(tok_ids)
    M, k = tok_ids.shape
    seg_expert = sorted(int(e) for e in S)
    perm: List[int] = []
    seg_off = [0]
    for e in seg_expert:
        for t in range(M):
            for j in range(k):
                if int(tok_ids[t, j]) == e:
                    perm.append(t * k + j)
        seg_off.append(len(perm))
    return (np.asarray(seg_expert, dtype=np.int32), np.asarray(seg_off, dtype=np.int32),
            np.asarray(perm, dtype=np.int32))


# --------------------------------------------------------------------------- experts
def silu(z):
    z = _f64(z)
    return z / (1.0 + np.exp(-z))


def expert(x, w_gate_e, w_up_e, w_down_e) -> np.ndarray:
    """E_i(x) = W_down ( silu(W_gate x) * (W_up x) ); W_gate, W_up [F, d], W_down [d, F]."""
    x = _f64(x)
    a = silu(_f64(w_gate_e) @ x) * (_f64(w_up_e) @ x)
    return _f64(w_down_e) @ a


class _ExpertBank:
    """fp64 copies of expert weights, converted on first use (memory only, no maths)."""

    def __init__(self, w_gate, w_up, w_down):
        self._w = (w_gate, w_up, w_down)
        self._cache: Dict[int, Tuple[np.ndarray, np.ndarray, np.ndarray]] = {}

    def get(self, e: int):
        if e not in self._cache:
            self._cache[e] = tuple(_f64(m[e]) for m in self._w)
        return self._cache[e]


def combine(h, tok_ids, tok_w, w_gate, w_up, w_down, tokens: Optional[Sequence[int]] = None) -> np.ndarray:
    """out[t] = sum over t's surviving slots, in slot order, of weight * E_i(h_t).

    A token with no surviving expert gets exact zeros.  ``tokens`` limits the
    evaluation to some rows (the others stay zero).
    """
    h = _f64(h)
    tok_ids = np.asarray(tok_ids)
    M, k = tok_ids.shape
    bank = _ExpertBank(w_gate, w_up, w_down)
    out = np.zeros((M, h.shape[1]), dtype=np.float64)
    for t in (range(M) if tokens is None else tokens):
        for j in range(k):
            e = int(tok_ids[t, j])
            if e < 0:
                continue
            out[t] = out[t] + float(tok_w[t][j]) * expert(h[t], *bank.get(e))
    return out


# --------------------------------------------------------------------------- Algorithm 1
def budget(g, topk_ids, topk_w, B: int, policy: int, k: int, renorm: bool,
           ext_shortlist: Optional[Sequence[int]] = None):
    """Stages 2-3 of Algorithm 1 without the expert maths.

    Returns a dict with scores, S (rank order), tok_ids, tok_w, seg_expert,
    seg_off, perm.  ``ext_shortlist`` replaces the router-based ranking by a
    shortlist fixed elsewhere (e.g. a static ranking, Eq. (4)).
    """
    s = aggregate_scores(g)
    S = list(ext_shortlist) if ext_shortlist is not None else shortlist(s, B)
    if policy == TRUNCATE:
        tok_ids, tok_w = restrict_truncation(topk_ids, topk_w, S)
    elif policy == SUBSTITUTE:
        tok_ids, tok_w = restrict_substitution(g, S, k, renorm)
    else:
        raise ValueError("unknown policy")
    seg_expert, seg_off, perm = segments(tok_ids, S)
    return dict(scores=s, S=np.asarray(S, dtype=np.int32), tok_ids=tok_ids, tok_w=tok_w,
                seg_expert=seg_expert, seg_off=seg_off, perm=perm)


def layer_forward(h, weights: Dict[str, np.ndarray], k: int, renorm: bool, B: int, policy: int,
                  tokens: Optional[Sequence[int]] = None, ext_shortlist: Optional[Sequence[int]] = None,
                  gate: str = SOFTMAX):
    """Algorithm 1 end to end for one layer.  Returns a dict of every intermediate and ``out``."""
    g, topk_ids, topk_w = route(h, weights["w_router"], weights.get("b_router"), k, renorm, gate)
    r = budget(g, topk_ids, topk_w, B, policy, k, renorm, ext_shortlist)
    r.update(probs=g, topk_ids=topk_ids, topk_w=topk_w, union=expert_union(topk_ids))
    r["loaded"] = sorted({int(e) for e in r["tok_ids"].ravel() if e >= 0})
    r["out"] = combine(h, r["tok_ids"], r["tok_w"], weights["w_gate"], weights["w_up"], weights["w_down"], tokens)
    return r


def unbudgeted_forward(h, weights: Dict[str, np.ndarray], k: int, renorm: bool,
                       tokens: Optional[Sequence[int]] = None, gate: str = SOFTMAX) -> np.ndarray:
    """Eq. (2): the standard MoE output over each token's natural top-k."""
    _, ids, w = route(h, weights["w_router"], weights.get("b_router"), k, renorm, gate)
    return combine(h, ids, w, weights["w_gate"], weights["w_up"], weights["w_down"], tokens)


def decision_margins(g, B: int, k: int, S: Optional[Sequence[int]] = None) -> Dict[str, float]:
    """Smallest gaps at the decision boundaries (for judging how safe ids are from rounding).

    ``topk``: min over tokens of adjacent gaps among the k+1 largest g;
    ``score``: min adjacent gap among the B+1 largest aggregate scores;
    ``sub``: (if S given) min over tokens of adjacent gaps among the k+1 largest g inside S.
    """
    g = _f64(g)
    res = {"topk": np.inf, "score": np.inf, "sub": np.inf}
    for t in range(g.shape[0]):
        v = sorted(g[t], reverse=True)[:k + 1]
        res["topk"] = min(res["topk"], min(a - b for a, b in zip(v, v[1:])))
        if S is not None:
            v = sorted((g[t][i] for i in S), reverse=True)[:k + 1]
            if len(v) > 1:
                res["sub"] = min(res["sub"], min(a - b for a, b in zip(v, v[1:])))
    v = sorted(aggregate_scores(g), reverse=True)[:B + 1]
    if len(v) > 1:
        res["score"] = min(a - b for a, b in zip(v, v[1:]))
    return {key: float(val) for key, val in res.items()}


# --------------------------------------------------------------------------- layer stack
def rms_scale(h) -> np.ndarray:
    """x[t] = h[t] / sqrt(mean_j h[t, j]^2): every row scaled to unit root-mean-square (no learned gain)."""
    h = _f64(h)
    x = np.empty_like(h)
    for t in range(h.shape[0]):
        x[t] = h[t] / np.sqrt(np.dot(h[t], h[t]) / h.shape[1])
    return x


def layer_stack(h, layers, k: int, renorm: bool, B: int, policy: int, store_fn=None, pre_norm: bool = False,
                gate: str = SOFTMAX):
    """Consecutive MoE layers joined by the residual connection: h <- h + MoE_S(x).

    ``pre_norm=False``: x = h, the recurrence as the layer-stack workload words it.  ``pre_norm=True``: x = h scaled
    row by row to unit root-mean-square (``rms_scale``) while the residual stream itself stays unscaled - the
    stack driver's guard against the hidden scale squaring from layer to layer (a SwiGLU expert is quadratic in the
    scale of its input).  ``layers`` yields one weight dict per layer.  ``store_fn`` (optional) rounds the MoE input
    and the running hidden state to their storage format.  Returns the final hidden state and the per-layer results
    (each with its MoE input under ``"x"``).
    """
    h = _f64(h)
    results = []
    for weights in layers:
        x = rms_scale(h) if pre_norm else h
        if store_fn is not None:
            x = _f64(store_fn(x))
        r = layer_forward(x, weights, k, renorm, B, policy, gate=gate)
        r["x"] = x
        results.append(r)
        h = h + r["out"]
        if store_fn is not None:
            h = _f64(store_fn(h))
    return h, results
