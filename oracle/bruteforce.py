"""Second, independent acceptance routine for tiny trees — TEST INFRASTRUCTURE ONLY.

Enumerates every root-to-leaf path of the draft tree, counts how many leading draft
tokens on it the target would have produced greedily (paper Section 3.1 at temperature
0: a token survives iff it equals the argmax at its parent), and keeps the longest
accepted prefix. Written separately from oracle.c's index-order walk, in another
language and by another route, so the two can check each other.
"""
from __future__ import annotations


def accept_bruteforce(amax, draft, parent):
    """Returns (accepted_len, path list root..best, bonus)."""
    T = len(parent)
    kids = {i: [] for i in range(T)}
    for i in range(1, T):
        kids[int(parent[i])].append(i)
    leaves = [i for i in range(T) if not kids[i]]
    best_prefix = [0]
    for leaf in leaves:
        chain = []
        j = leaf
        while j != -1:
            chain.append(j)
            j = int(parent[j])
        chain.reverse()                      # root .. leaf
        good = [chain[0]]
        for a, b in zip(chain[:-1], chain[1:]):
            if int(draft[b]) != int(amax[a]):
                break
            good.append(b)
        if len(good) > len(best_prefix) or (len(good) == len(best_prefix) and good[-1] < best_prefix[-1]):
            best_prefix = good
    return len(best_prefix) - 1, best_prefix, int(amax[best_prefix[-1]])


def reachability_mask(parent):
    """Ancestor-or-self bit masks by transitive closure of the child→parent relation
    (Warshall), a different route from walking parent pointers."""
    T = len(parent)
    reach = [[i == j for j in range(T)] for i in range(T)]
    for i in range(1, T):
        reach[i][int(parent[i])] = True
    for k in range(T):
        for i in range(T):
            if reach[i][k]:
                for j in range(T):
                    if reach[k][j]:
                        reach[i][j] = True
    return [sum(1 << j for j in range(T) if reach[i][j]) for i in range(T)]


def sample_output_distribution(p_rows, draft, parent, max_tokens=None):
    """Exact distribution of the token sequence that stochastic tree acceptance emits, by
    enumerating every outcome of its accept / reject decisions with rational-free float64
    probabilities. p_rows[i] is the target distribution at node i (a list summing to 1).
    Returns {tuple of emitted tokens (accepted draft tokens, then the bonus): probability}.

    Written from the rule itself (try the children in node order, accept child c with the
    residual probability of its token, otherwise delete that token and renormalise; when no
    child is accepted draw the bonus from what is left) and independent of oracle.c; the
    tests compare this distribution with the product of target conditionals."""
    T = len(parent)
    kids = {i: [c for c in range(i + 1, T) if int(parent[c]) == i] for i in range(T)}
    out = {}

    def visit(node, prefix, prob):
        resid = list(p_rows[node])
        mass = prob                                   # probability of standing here with this residual
        for c in kids[node]:
            x = int(draft[c])
            tot = sum(resid)
            r = resid[x] / tot if tot > 0 and 0 <= x < len(resid) else 0.0
            if r > 0:
                visit(c, prefix + (x,), mass * r)
                mass *= (1.0 - r)
                resid[x] = 0.0
        tot = sum(resid)
        if mass > 0 and tot > 0:
            for y, w in enumerate(resid):
                if w > 0:
                    key = prefix + (y,)
                    out[key] = out.get(key, 0.0) + mass * w / tot

    visit(0, (), 1.0)
    return out


def best_closed_subset(scores, parent, N):
    """Exhaustive search for the draft tree's final selection (tiny inputs only): among all sets
    of min(N, M) candidates that contain the parent of each member, the one with the largest
    total probability sum(exp(score)). Returns the sorted tuple of candidate indices. A route
    that never sorts by score, to check the oracle's "take the N best scores" against what that
    rule is claimed to achieve."""
    import itertools
    import math
    M = len(scores)
    n = min(N, M)
    best, best_val = None, -1.0
    for sub in itertools.combinations(range(M), n):
        s = set(sub)
        if any(parent[c] >= 0 and parent[c] not in s for c in sub):
            continue
        val = sum(math.exp(scores[c]) for c in sub)
        if val > best_val:
            best, best_val = sub, val
    return best


def expand_frontier_bruteforce(logits_rows, cum_in, K):
    """One expansion step by full sorting in Python (independent of oracle.c): returns
    (tokens, scores, kept candidate indices ascending)."""
    import math
    toks, scs = [], []
    for f, row in enumerate(logits_rows):
        m = max(row)
        lse = m + math.log(math.fsum(math.exp(x - m) for x in row))
        order = sorted(range(len(row)), key=lambda j: (-row[j], j))[:K]
        toks += order
        scs += [cum_in[f] + (row[j] - lse) for j in order]
    keep = sorted(sorted(range(len(scs)), key=lambda c: (-scs[c], c))[:K])
    return toks, scs, keep
