"""Greedy best-first search over the key graph (test oracle; see package header).

Sec. 2.4 describes proximity-graph search as a greedy walk that moves to the most
similar vectors at each hop; Algorithm 1 calls it VectorSearch(q). The paper fixes
nothing else, so the walk below is the usual bounded-beam best-first search with
this build's determinism choices:

  state   visited set; beam of at most `ef` (score, id, expanded?) entries kept under
          the total order of mips.py (score descending, id ascending).
  start   visited = {entry}; beam = {entry}. With a seed set (below) instead:
          visited = the seeds, beam = the best `ef` of them, none expanded.
  step    take the `expand` best not-yet-expanded beam entries (all of them if fewer);
          stop if there are none. Mark them expanded. Gather their adjacency rows; the
          new candidates are the distinct valid neighbours not yet visited. Mark them
          visited, score them, add them to the beam, and keep the best `ef`.
  result  walk the final beam best-first, skip ids in the static set, take `topk`.

Seed set. The paper does not say where a walk starts. A single entry point makes the
first hops of every walk the same climb from the graph's root towards the query; the walk
may instead start from the `n_seeds` keys nearest the root, all scored at once:
`backbone_seeds` lists them from the graph alone, breadth first over the binary tree that
the first two slots of every adjacency row span from the entry point. For a graph made by
projection.py those slots hold the popularity heap, so the seeds are the n_seeds keys that
appear in the most KNN lists of the prefill queries, in that order, the entry point first.
seeds = [entry] is the single-entry start.

With expand = 1 this is the textbook loop; a larger width trades a few extra
expansions for fewer dependent steps. The beam content after a step does not depend
on the order candidates are inserted in (top-ef of a union), so it is well defined.

Scores are the plain inner product of Sec. 2.4 in float64 (`scores_f64`) unless the
caller passes another `score_fn`. A device kernel scores in float32, so where two float64
scores nearly coincide it may order them the other way; to let a test tell such a case from
a real difference, the walk reports `min_gap`: the smallest relative gap
|a - b| / max(|a|, |b|) between two scores whose order decided something (which entries a
step expands, which entries fall off the beam, the order and the cut of the result). A walk
whose min_gap is above a kernel's score error takes the same decisions in that kernel.
Bit-identical key rows score identically in any arithmetic, so a gap of exactly zero between
two such rows is decided by the ids and is not counted.

`score32` is an opt-in `score_fn`: the same inner product in float32, summed in one fixed
order (16 contiguous chunks summed left to right, product rounded then added, the 16 chunk
sums added pairwise in a balanced tree over adjacent chunks). With it the walk's decisions
are taken in float32 and can be compared bit for bit with a float32 implementation that
adds in that order. It is pinned against the float64 inner product in the tests.
"""
import numpy as np

F32 = np.float32


def score32(q, Krows):
    """Inner products <q, k> for each row of Krows in the fixed float32 order above.
    q: [d], Krows: [n][d] (values exactly representable in float32). d % 16 == 0."""
    q = np.asarray(q, F32)
    Kr = np.asarray(Krows, F32)
    n, d = Kr.shape
    if d % 16:
        raise ValueError("d must be a multiple of 16")
    c = d // 16
    part = np.zeros((n, 16), F32)
    for lane in range(16):
        acc = np.zeros(n, F32)
        for i in range(c):
            prod = (Kr[:, lane * c + i] * q[lane * c + i]).astype(F32)
            acc = (acc + prod).astype(F32)
        part[:, lane] = acc
    while part.shape[1] > 1:
        part = (part[:, 0::2] + part[:, 1::2]).astype(F32)
    return part[:, 0]


def _sort_beam(beam):
    beam.sort(key=lambda e: (-e[0], e[1]))


def scores_f64(q, Krows):
    """<q, k> for each row of Krows, float64: the plain definition (Sec. 2.4)."""
    return np.asarray(Krows, np.float64) @ np.asarray(q, np.float64)


def _rel_gap(a, b):
    m = max(abs(a), abs(b))
    return abs(a - b) / m if m > 0 else 0.0


def backbone_seeds(adj, entry, n_seeds):
    """The first `n_seeds` positions, breadth first, of the binary tree spanned from `entry`
    by slots 0 and 1 of every adjacency row (position p has its children at positions 2p + 1
    and 2p + 2). Positions without a node (a -1 slot, or below one) and nodes already listed
    are left out; the order of first occurrence is kept. Returns int64 ids, entry first."""
    adj = np.asarray(adj)
    if n_seeds < 1:
        raise ValueError("n_seeds must be positive")
    pos = [-1] * n_seeds
    pos[0] = int(entry)
    for p in range(n_seeds):
        if pos[p] < 0:
            continue
        for slot in (0, 1):
            c = 2 * p + 1 + slot
            if c < n_seeds and slot < adj.shape[1]:
                pos[c] = int(adj[pos[p], slot])
    seen, out = set(), []
    for i in pos:
        if i >= 0 and i not in seen:
            seen.add(i)
            out.append(i)
    return np.array(out, np.int64)


def greedy_search(q, K, adj, entry, ef, topk, expand=1, exclude=None, score_fn=None, seeds=None):
    """Returns (ids int32 [topk] padded with -1, stats dict) with stats =
    {n_visited, n_expanded, n_iters, n_returned, beam: [(score, id)] best-first, min_gap}.
    score_fn(q, rows) -> scores; default float64 inner products. seeds: distinct ids the walk
    starts from (default: the entry point alone)."""
    if ef < topk or ef < 1 or topk < 1 or expand < 1:
        raise ValueError("need ef >= topk >= 1 and expand >= 1")
    score_fn = scores_f64 if score_fn is None else score_fn
    K = np.asarray(K)
    adj = np.asarray(adj)
    excl = set(int(i) for i in exclude) if exclude is not None else set()
    gaps = [np.inf]

    def decided(x, y):
        # the order of beam entries x, y decided something: note how close their scores are
        if x[0] == y[0] and np.array_equal(K[x[1]], K[y[1]]):
            return
        gaps.append(_rel_gap(x[0], y[0]))

    start = [int(entry)] if seeds is None else [int(i) for i in seeds]
    if not start or len(set(start)) != len(start):
        raise ValueError("seeds must be distinct and not empty")
    visited = set(start)
    beam = [[float(s), i, False] for s, i in zip(score_fn(q, K[start]), start)]
    _sort_beam(beam)
    if len(beam) > ef:
        decided(beam[ef - 1], beam[ef])
    del beam[ef:]
    n_expanded = n_iters = 0
    while True:
        unexpanded = [e for e in beam if not e[2]]         # beam is kept best-first
        pick = unexpanded[:expand]
        if not pick:
            break
        if len(unexpanded) > expand:
            decided(unexpanded[expand - 1], unexpanded[expand])
        n_iters += 1
        new = []
        for e in pick:
            e[2] = True
            n_expanded += 1
            for n in adj[e[1]]:
                n = int(n)
                if n >= 0 and n not in visited:
                    visited.add(n)
                    new.append(n)
        if new:
            sc = score_fn(q, K[new])
            beam.extend([float(s), n, False] for s, n in zip(sc, new))
        _sort_beam(beam)
        if len(beam) > ef:
            decided(beam[ef - 1], beam[ef])
        del beam[ef:]
    eligible = [e for e in beam if e[1] not in excl]
    for x, y in zip(eligible[:topk], eligible[1:topk + 1]):
        decided(x, y)
    res = [e[1] for e in eligible][:topk]
    ids = np.full(topk, -1, np.int32)
    ids[:len(res)] = res
    return ids, dict(n_visited=len(visited), n_expanded=n_expanded, n_iters=n_iters,
                     n_returned=len(res), beam=[(e[0], e[1]) for e in beam], min_gap=float(min(gaps)))
