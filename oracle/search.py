"""Greedy best-first search over the key graph (test oracle; see package header).

Sec. 2.4 describes proximity-graph search as a greedy walk that moves to the most
similar vectors at each hop; Algorithm 1 calls it VectorSearch(q). The paper fixes
nothing else, so the walk below is the usual bounded-beam best-first search with
this build's determinism choices:

  state   visited set; beam of at most `ef` (score, id, expanded?) entries kept under
          the total order of mips.py (score descending, id ascending).
  start   visited = {entry}; beam = {entry}.
  step    take the `expand` best not-yet-expanded beam entries (all of them if fewer);
          stop if there are none. Mark them expanded. Gather their adjacency rows; the
          new candidates are the distinct valid neighbours not yet visited. Mark them
          visited, score them, add them to the beam, and keep the best `ef`.
  result  walk the final beam best-first, skip ids in the static set, take `topk`.

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


def greedy_search(q, K, adj, entry, ef, topk, expand=1, exclude=None, score_fn=None):
    """Returns (ids int32 [topk] padded with -1, stats dict) with stats =
    {n_visited, n_expanded, n_iters, n_returned, beam: [(score, id)] best-first, min_gap}.
    score_fn(q, rows) -> scores; default float64 inner products."""
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

    visited = {int(entry)}
    s0 = float(score_fn(q, K[[entry]])[0])
    beam = [[s0, int(entry), False]]
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
