"""Brute-force statement of the method for TINY inputs, in exact rational
arithmetic, used only to pin the C++ oracle.

Written from the definitions, not from the oracle: matches are a literal
set-builder over every (j, e) (Eq. 3 of the paper), candidates are explicit
token sequences, edge weights are Eq. 5 evaluated with fractions.Fraction for
a real-valued alpha, and the greedy rule is evaluated on those rationals.
"""
from collections import defaultdict
from fractions import Fraction
from functools import lru_cache


def quant(p):
    """Probability as a multiple of 1/65536 (Python round() is half-to-even)."""
    if p != p:
        return 0
    return max(0, min(65536, round(float(p) * 65536.0)))


def within_one_edit(a, b):
    """Levenshtein(a, b) <= 1 without dynamic programming: equal, one substitution, or one
    string is the other with a single element removed."""
    a, b = tuple(a), tuple(b)
    if a == b:
        return True
    if len(a) == len(b):
        return sum(x != y for x, y in zip(a, b)) == 1
    if len(a) > len(b):
        a, b = b, a
    return len(b) - len(a) == 1 and any(b[:x] + b[x + 1:] == a for x in range(len(b)))


@lru_cache(maxsize=None)
def lev(a, b):
    """Levenshtein distance by its recursive definition (tuples)."""
    if not a:
        return len(b)
    if not b:
        return len(a)
    return min(lev(a[1:], b[1:]) + (a[0] != b[0]), lev(a[1:], b) + 1, lev(a, b[1:]) + 1)


def match_set(paths, i, k, eps=0, include_self=False):
    """include_self: path i's own history is searched too (a match still needs a successor, so
    the query's own occurrence at the end of path i never counts)."""
    yi = paths[i]
    q = min(k, len(yi))
    if q == 0:
        return q, set()
    suffix = tuple(yi[len(yi) - q:])
    searched = [(j, yj) for j, yj in enumerate(paths) if j != i or include_self]
    if eps == 0:
        return q, {(j, e) for j, yj in searched
                   for e in range(q, len(yj)) if tuple(yj[e - q:e]) == suffix}
    near = within_one_edit if eps == 1 else (lambda a, b: lev(tuple(a), tuple(b)) <= eps)
    return q, {(j, e) for j, yj in searched for e in range(len(yj))
               if any(near(suffix, yj[e - l:e]) for l in range(0, e + 1))}


def backed_off_k(paths, i, k, eps=0, include_self=False):
    """Query back-off: the largest query length <= k whose match set is not empty (k itself if
    there is none: the draft is empty either way)."""
    for shorter in range(min(k, len(paths[i])), 0, -1):
        if match_set(paths, i, shorter, eps, include_self)[1]:
            return shorter
    return k


def candidates(paths, probs, i, k, L, eps=0, include_self=False):
    """Each candidate = [(predecessor, token, prob_fraction), ...] of length <= L.  The
    predecessor of a candidate's first token is the query's last token (the DAG's root)."""
    _, M = match_set(paths, i, k, eps, include_self)
    out = []
    for (j, e) in M:
        seq = []
        for t in range(e, min(e + L, len(paths[j]))):
            p = Fraction(quant(probs[j][t]), 65536) if probs is not None else Fraction(1)
            seq.append((paths[i][-1] if t == e else paths[j][t - 1], paths[j][t], p))
        out.append(seq)
    return out


def edge_tables(paths, probs, i, k, L, eps=0, include_self=False):
    """{(d, u, v): [count, prob_sum_fraction]} with d = 1..L."""
    E = defaultdict(lambda: [0, Fraction(0)])
    for seq in candidates(paths, probs, i, k, L, eps, include_self):
        for d, (u, v, p) in enumerate(seq, start=1):
            E[(d, u, v)][0] += 1
            E[(d, u, v)][1] += p
    return dict(E)


def draft(paths, probs, i, k, L, alpha=Fraction(1), score_mode=0, eps=0, include_self=False, backoff=False):
    """Returns (tokens, scores) with scores as exact Fractions."""
    alpha = Fraction(alpha)
    if backoff:
        k = backed_off_k(paths, i, k, eps, include_self)
    E = edge_tables(paths, probs, i, k, L, eps, include_self)
    if not E:
        return [], []

    def w(cs):
        return alpha * cs[1] + (1 - alpha) * cs[0]

    cur = paths[i][-1]
    toks, scores = [], []
    for d in range(1, L + 1):
        succ = sorted(v for (dd, u, v) in E if dd == d and u == cur)
        if not succ:
            break
        def score(v):
            if score_mode == 1:
                return w(E[(d, cur, v)])
            return sum(w(cs) for (dd, u, vv), cs in E.items() if dd == d and vv == v)
        best = max(score(v) for v in succ)
        v_star = min(v for v in succ if score(v) == best)
        toks.append(v_star)
        scores.append(best)
        cur = v_star
    return toks, scores


def accept(draft_tokens, target):
    a = 0
    for x, y in zip(draft_tokens, target):
        if x != y:
            break
        a += 1
    return a


def tree_draft(paths, probs, i, k, L, alpha=Fraction(1), eps=0, include_self=False, backoff=False):
    """The ablation's tree pool: an explicit prefix tree (nested dicts) of the candidates'
    continuations; each node carries [count, prob_sum] of the candidates through it; the draft
    is the greedy descent to the heaviest child (ties: lowest token id)."""
    alpha = Fraction(alpha)
    if backoff:
        k = backed_off_k(paths, i, k, eps, include_self)
    root = {}                                   # token -> [count, prob_sum, children]
    for seq in candidates(paths, probs, i, k, L, eps, include_self):
        node = root
        for (_, v, p) in seq:
            entry = node.setdefault(v, [0, Fraction(0), {}])
            entry[0] += 1
            entry[1] += p
            node = entry[2]
    toks, scores = [], []
    node = root
    while node and len(toks) < L:
        weight = {v: alpha * ent[1] + (1 - alpha) * ent[0] for v, ent in node.items()}
        best = max(weight.values())
        v_star = min(v for v in weight if weight[v] == best)
        toks.append(v_star)
        scores.append(best)
        node = node[v_star][2]
    return toks, scores


def list_draft(paths, probs, i, k, L, alpha=Fraction(1), eps=0, include_self=False, backoff=False):
    """The ablation's list pool: the continuation of the single candidate whose tokens'
    weights (alpha * p + (1 - alpha) each) add up to the most; ties: first in (j, e) order."""
    alpha = Fraction(alpha)
    if backoff:
        k = backed_off_k(paths, i, k, eps, include_self)
    _, M = match_set(paths, i, k, eps, include_self)
    best_key, best = None, ([], [])
    for (j, e) in sorted(M):
        toks = list(paths[j][e:e + L])
        ws = [alpha * (Fraction(quant(probs[j][t]), 65536) if probs is not None else Fraction(1)) + (1 - alpha)
              for t in range(e, e + len(toks))]
        if best_key is None or sum(ws) > best_key:
            best_key, best = sum(ws), (toks, ws)
    return best
