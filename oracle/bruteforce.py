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
