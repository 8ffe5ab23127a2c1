"""Projection of the query->key KNN lists into a key-key proximity graph
(test oracle; see package header).

Sec. 3.2 states the step in one sentence: key vectors that are connected to the
same query vectors are linked, so that keys which look close from the queries'
point of view become neighbours and the query vectors can be dropped. Degree
bound, neighbour choice, entry point and connectivity are not given. The reading
implemented here (everything below is integer arithmetic on the KNN lists):

 1. pop(i)  = number of KNN lists that contain key i.
    c(a,b)  = number of KNN lists that contain both a and b (a != b): the number of
              query vectors both keys are connected to.
 2. pi      = all keys ordered by (pop descending, id ascending); entry = pi[0].
 3. For a key a with pop(a) >= 1 its candidates are the keys b with c(a,b) >= 1,
    ranked by the Jaccard overlap of their query sets
          J(a,b) = c / (pop(a) + pop(b) - c)           (descending, compared exactly
    as fractions), ties by larger c, then by lower id.
 4. Backbone: the key at position t of pi gets out-edges to pi[2t+1] and pi[2t+2]
    where they exist (an implicit binary heap over popularity). Every key has exactly
    one backbone in-edge, so every key is reachable from `entry`.
 5. Row a of the adjacency = its backbone children (in that order), followed by its
    ranked candidates that are not already in the row, until `deg` entries; the rest
    is padded with -1. No self-loops, no duplicates.

Why Jaccard and not the raw count: when the queries share a strong common component,
a few keys sit in almost every list and the raw count makes every key choose the same
few hubs; the overlap ratio ranks by what is specific to the pair.

PARITY UNPINNED by the paper for this function (it prints no worked example).
"""
from functools import cmp_to_key

import numpy as np


def popularity(L, N):
    """pop(i): how many lists contain key i (each list holds distinct ids)."""
    return np.bincount(np.asarray(L).ravel().astype(np.int64), minlength=N).astype(np.int64)


def popularity_order(pop):
    """pi: key ids by (pop descending, id ascending)."""
    N = len(pop)
    return np.array(sorted(range(N), key=lambda i: (-int(pop[i]), i)), dtype=np.int64)


def cooccurrence_of(L, a, members=None):
    """{b: c(a,b)} for one key a. `members` (optional) = indices of lists holding a."""
    L = np.asarray(L)
    if members is None:
        members = [j for j in range(L.shape[0]) if a in L[j]]
    if len(members) == 0:
        return {}
    ids, cnt = np.unique(L[np.asarray(members, np.int64)], return_counts=True)
    return {int(b): int(c) for b, c in zip(ids, cnt) if int(b) != a}


def _closer(pop_a, pop):
    """Comparator on (b, c) candidate tuples implementing step 3's order exactly."""
    def cmp(x, y):
        bx, cx = x
        by, cy = y
        ux = pop_a + int(pop[bx]) - cx
        uy = pop_a + int(pop[by]) - cy
        lhs, rhs = cx * uy, cy * ux          # J_x > J_y  <=>  cx*uy > cy*ux
        if lhs != rhs:
            return -1 if lhs > rhs else 1
        if cx != cy:
            return -1 if cx > cy else 1
        return -1 if bx < by else (1 if bx > by else 0)
    return cmp


def ranked_candidates(L, a, pop, members=None):
    """Step 3 for one key: candidate ids best-first."""
    c = cooccurrence_of(L, a, members)
    items = sorted(c.items(), key=cmp_to_key(_closer(int(pop[a]), pop)))
    return [b for b, _ in items]


def adjacency_row(L, a, pop, pi_pos, pi, deg, members=None):
    """Step 5 for one key a: its `deg` out-neighbours (padded with -1)."""
    N = len(pop)
    row = []
    t = int(pi_pos[a])
    for ch in (2 * t + 1, 2 * t + 2):
        if ch < N and len(row) < deg:
            row.append(int(pi[ch]))
    if pop[a] >= 1:
        for b in ranked_candidates(L, a, pop, members):
            if len(row) >= deg:
                break
            if b not in row:
                row.append(b)
    return row + [-1] * (deg - len(row))


def project(L, N, deg, rows=None):
    """KNN lists L [M][knn] -> (adj int32 [N][deg], entry). With `rows` given, only
    those adjacency rows are computed (the others are left as -1); used to check a
    sample of rows at sizes where the whole graph would take too long here."""
    L = np.asarray(L)
    if deg < 2:
        raise ValueError("deg must be at least 2 (two backbone slots)")
    pop = popularity(L, N)
    pi = popularity_order(pop)
    pi_pos = np.empty(N, np.int64)
    pi_pos[pi] = np.arange(N)
    members = {}
    for j in range(L.shape[0]):
        for i in L[j]:
            members.setdefault(int(i), []).append(j)
    adj = -np.ones((N, deg), np.int32)
    for a in (range(N) if rows is None else rows):
        adj[a] = adjacency_row(L, int(a), pop, pi_pos, pi, deg, members.get(int(a), []))
    return adj, int(pi[0])
