"""CPU oracle for the per-chunk streaming sparse-attention step of Ltri-LLM.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
library is checked against.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path never does.  It shares no
code with the HIP path and imports nothing from it.  All arithmetic is fp64
numpy; a library matmul / cumsum / sort may serve as a step, nothing is
blocked, fused or reordered beyond what the paper's definitions state.

Notation follows the paper: N (here L) tokens of a chunk, H heads summed,
A the causal attention map (Eq. 1-3), S*_{xy} / S_{xy} the Triangle-Attention
score of the span [x, y] (Eq. 4 / Eq. 5), theta the map threshold, phi the
NMS IoU threshold, index (representative) vectors K^R / Q^R (Sec. 3.3),
sim_{ij} (Eq. 8), Top-K retrieval (Eq. 9), and the attended set
initial | retrieved | window | current (Sec. 3.4, third step).

Readings taken where the paper is silent (each is listed in the design notes):
  * the map that is segmented is the appended chunk's own L x L causal map;
  * theta is an absolute per-head value (it sits inside the head sum in Eq. 5);
  * NMS boxes are 1-D token intervals, IoU on inclusive token counts;
  * kept intervals are turned into a tiling by cutting at all their end points;
  * the representative vector of a span is the mean of its rows (mean pooling,
    Sec. 3.3.1); by bilinearity Eq. 8 only needs one vector per span;
  * retrieval works on spans under a token budget (longest fitting prefix of
    the score order), not on fixed 128-token blocks;
  * LOGIT map kind (masked scaled scores without the softmax) exists next to
    the paper's SOFTMAX kind because row-normalised maps of planted keys do
    not carry mixed-length triangles.

Pinned by tests/test_oracle_pins.py (brute-force triple sums, ideal-map and
planted-key boundary recovery, NMS brute force, top-k vs full sort, the
select-everything == full causal attention invariant, brute-force softmax
attention, LSE-merge identity, decode == one-row prefill).
Dynamic index vectors (Sec. 3.3.2): votes, area ratios, Eq. 7 and the index
tokens are pinned by closed forms on constant keys (harmonic numbers), by the
row-sum identities of a softmax map, by Eq. 7's special values and by brute
force for the top-count choice and for Eq. 8's double sum.
Parity unpinned: the SOFTMAX map kind on planted keys has no ground truth for
which spans are "right"; it is pinned only through Eq. 4/5 and the NMS pins.
Likewise nothing outside this file says which tokens are the "right" index
tokens of a span: beyond the pins above that part is parity unpinned.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

MAP_SOFTMAX = 0
MAP_LOGIT = 1
REP_MEAN = 0
REP_DYNAMIC = 1


# ----------------------------------------------------------------------------
# rounding helper (representative vectors are stored in the stream's dtype)
# ----------------------------------------------------------------------------
def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values once, to nearest-even, to `dtype` ("f32" | "bf16" | "f64")."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f64":
        return x.copy()
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype == "bf16":
        m, e = np.frexp(x)                 # x = m * 2**e, 0.5 <= |m| < 1
        q = np.rint(m * 256.0) / 256.0     # keep 8 significant bits, ties to even
        return np.ldexp(q, e)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# step 1a: causal map of one chunk (Eq. 1-3), summed over the heads (Eq. 4)
# ----------------------------------------------------------------------------
def chunk_map(K: np.ndarray, Q: Optional[np.ndarray], kind: int) -> Tuple[np.ndarray, int]:
    """Head-summed lower-triangular map of one chunk for one KV head.

    K: [L, d] keys of the chunk.  Q: [G, L, d] queries of the KV head's group,
    or None, in which case the keys play the role of the queries (one head).
    Returns (M [L, L] with zeros above the diagonal, n_h = heads summed).
    """
    K = np.asarray(K, dtype=np.float64)
    L, d = K.shape
    Qs = K[None] if Q is None else np.asarray(Q, dtype=np.float64)
    n_h = Qs.shape[0]
    low = np.tril(np.ones((L, L), dtype=bool))           # mask P of Eq. 2
    M = np.zeros((L, L), dtype=np.float64)
    for g in range(n_h):
        z = (Qs[g] @ K.T) / math.sqrt(d)
        if kind == MAP_SOFTMAX:
            z = np.where(low, z, -np.inf)
            z = z - z.max(axis=1, keepdims=True)
            e = np.exp(z)
            a = e / e.sum(axis=1, keepdims=True)           # Eq. 1 restricted by Eq. 3
        elif kind == MAP_LOGIT:
            a = z
        else:
            raise ValueError(kind)
        M += np.where(low, a, 0.0)
    return M, n_h


# ----------------------------------------------------------------------------
# step 1b: Triangle-Attention score of every span (Eq. 4, Eq. 5)
# ----------------------------------------------------------------------------
def ta_scores(M: np.ndarray, theta: float, n_h: int) -> np.ndarray:
    """S[x, y] for 0 <= x <= y < L; entries with x > y are -inf.

    Second form of Eq. 4: rows 0..y, columns x..L-1 of the lower-triangular
    map, i.e. a cumulative sum from the right along each row followed by a
    cumulative sum down each column.  Eq. 5 subtracts theta on every cell of
    the mask inside the head sum, i.e. theta * n_h * (#cells of the triangle).
    """
    L = M.shape[0]
    R = np.cumsum(M[:, ::-1], axis=1)[:, ::-1]           # R[i, x] = sum_{j >= x} M[i, j]
    C = np.cumsum(R, axis=0)                             # C[y, x] = sum_{i <= y} R[i, x]
    x = np.arange(L)[:, None]
    y = np.arange(L)[None, :]
    n = y - x + 1
    tri = n * (n + 1) // 2
    S = C.T - theta * n_h * tri
    return np.where(x <= y, S, -np.inf)


# ----------------------------------------------------------------------------
# step 1c: candidate filter (appendix "NMS Input Filtration")
# ----------------------------------------------------------------------------
def antidiagonal_candidates(S: np.ndarray) -> List[Tuple[float, int, int]]:
    """Best-scoring span on each anti-diagonal x + y = s, kept only if its score is > 0.

    Ties go to the larger x (the shorter span)."""
    L = S.shape[0]
    out = []
    for s in range(2 * L - 1):
        x_lo = max(0, s - (L - 1))
        x_hi = s // 2
        xs = np.arange(x_lo, x_hi + 1)
        vals = S[xs, s - xs]
        best = vals.max()
        if not best > 0.0:
            continue
        x = int(xs[np.nonzero(vals == best)[0][-1]])
        out.append((float(best), x, s - x))
    return out


# ----------------------------------------------------------------------------
# step 1d: greedy NMS on 1-D intervals (Sec. 3.2)
# ----------------------------------------------------------------------------
def nms_1d(cands: Sequence[Tuple[float, int, int]], phi: float,
           max_keep: int = 0) -> List[Tuple[float, int, int]]:
    """Greedy non-maximum suppression.

    Candidates are visited by decreasing score (ties: smaller x, then smaller
    y).  A candidate is dropped when some already kept interval overlaps it
    with intersection > phi * union, both counted in tokens (inclusive ends);
    the comparison is done in fp32 with a single multiply so it can be
    reproduced exactly elsewhere.  `max_keep` > 0 stops after that many keeps.
    """
    order = sorted(cands, key=lambda c: (-c[0], c[1], c[2]))
    phi32 = np.float32(phi)
    kept: List[Tuple[float, int, int]] = []
    for (s, x, y) in order:
        ok = True
        for (_, a, b) in kept:
            inter = min(y, b) - max(x, a) + 1
            if inter <= 0:
                continue
            union = (y - x + 1) + (b - a + 1) - inter
            if np.float32(inter) > phi32 * np.float32(union):
                ok = False
                break
        if ok:
            kept.append((s, x, y))
            if max_keep and len(kept) >= max_keep:
                break
    return kept


def partition_from_kept(kept: Sequence[Tuple[float, int, int]], L: int, unit: int = 0, c0: int = 0
                        ) -> np.ndarray:
    """Cut [0, L) at every kept interval's x and y+1; returns the sorted cuts incl. 0 and L.
    unit > 0: the chunk starts at absolute position c0 and is also cut wherever a memory unit of
    `unit` tokens ends, so that every span lies inside one unit (Eq. 9 speaks of the spans of
    block b)."""
    cuts = {0, L}
    for (_, x, y) in kept:
        cuts.add(x)
        cuts.add(y + 1)
    if unit > 0:
        cuts.update(i for i in range(1, L) if (c0 + i) % unit == 0)
    return np.asarray(sorted(cuts), dtype=np.int64)


def map_quantile(M: np.ndarray, q: float) -> float:
    """The threshold as a percentile of the map (Sec. 4, "Hyperparameter Tuning": the typical
    theta is the 90th percentile): the value of rank floor(q (n - 1)) among the n cells on and
    below the diagonal of the head-summed map, in ascending order (nearest rank, no interpolation)."""
    M = np.asarray(M, np.float64)
    cells = np.sort(M[np.tril_indices(M.shape[0])])
    return float(cells[int(math.floor(q * (len(cells) - 1)))])


def segment_chunk(K: np.ndarray, Q: Optional[np.ndarray], kind: int, theta: float,
                  phi: float, max_keep: int = 0, z_perturb: Optional[np.ndarray] = None,
                  theta_quantile: float = 0.0, unit: int = 0, c0: int = 0) -> np.ndarray:
    """Boundaries (chunk-local, first 0, last L) of the spans of one chunk (Sec. 3.4, first step).
    theta_quantile > 0: theta is that percentile of the head-summed map's cells (then `theta` is
    ignored); the value applies per head-summed cell, i.e. Eq. 5's theta is it over n_h."""
    M, n_h = chunk_map(K, Q, kind)
    if z_perturb is not None:
        M = M * (1.0 + z_perturb)
    if theta_quantile > 0.0:
        theta = map_quantile(M, theta_quantile) / n_h
    S = ta_scores(M, theta, n_h)
    cands = antidiagonal_candidates(S)
    kept = nms_1d(cands, phi, max_keep)
    return partition_from_kept(kept, K.shape[0], unit, c0)


def segmentation_is_stable(K: np.ndarray, Q: Optional[np.ndarray], kind: int, theta: float,
                           phi: float, max_keep: int = 0, rel: float = 2.0 ** -18,
                           draws: int = 2, seed: int = 0, theta_quantile: float = 0.0,
                           unit: int = 0, c0: int = 0) -> bool:
    """Audit of one chunk: do the boundaries survive relative perturbations of every map
    cell that are ~32x larger than fp32 rounding?  Bit-exact parity with an fp32
    map is only asserted on chunks that pass."""
    base = segment_chunk(K, Q, kind, theta, phi, max_keep, theta_quantile=theta_quantile, unit=unit, c0=c0)
    rng = np.random.default_rng(seed)
    L = K.shape[0]
    for _ in range(draws):
        p = rng.uniform(-rel, rel, size=(L, L))
        b = segment_chunk(K, Q, kind, theta, phi, max_keep, z_perturb=p, theta_quantile=theta_quantile,
                          unit=unit, c0=c0)
        if len(b) != len(base) or np.any(b != base):
            return False
    return True


def segmentation_reachable(K: np.ndarray, Q: Optional[np.ndarray], kind: int, theta: float,
                           phi: float, target: Sequence[int], max_keep: int = 0, rel: float = 2.0 ** -16,
                           draws: int = 32, seed: int = 1, theta_quantile: float = 0.0,
                           unit: int = 0, c0: int = 0) -> bool:
    """Validity check for a chunk that fails the audit above: is `target` (boundaries found by an
    implementation whose map cells carry a relative error below `rel`) what this procedure yields
    for SOME map within that error?  True if the unperturbed map or one of `draws` random relative
    perturbations bounded by `rel` gives exactly `target`.  A tiling that no admissible map
    produces is a bug, not a near-tie."""
    target = [int(t) for t in target]
    base = segment_chunk(K, Q, kind, theta, phi, max_keep, theta_quantile=theta_quantile, unit=unit, c0=c0)
    if [int(t) for t in base] == target:
        return True
    rng = np.random.default_rng(seed)
    L = K.shape[0]
    for _ in range(draws):
        p = rng.uniform(-rel, rel, size=(L, L))
        b = segment_chunk(K, Q, kind, theta, phi, max_keep, z_perturb=p, theta_quantile=theta_quantile,
                          unit=unit, c0=c0)
        if [int(t) for t in b] == target:
            return True
    return False


# ----------------------------------------------------------------------------
# representative vectors (mean pooling, Sec. 3.3.1) and similarity (Eq. 8)
# ----------------------------------------------------------------------------
def span_means(X: np.ndarray, bounds: np.ndarray, dtype: str) -> np.ndarray:
    """Mean of the rows of X [L, d] over each span [bounds[s], bounds[s+1]); rounded once to dtype."""
    X = np.asarray(X, dtype=np.float64)
    out = np.empty((len(bounds) - 1, X.shape[1]), dtype=np.float64)
    for s in range(len(bounds) - 1):
        a, b = int(bounds[s]), int(bounds[s + 1])
        out[s] = X[a:b].sum(axis=0) / float(b - a)
    return round_to_dtype(out, dtype)


# ----------------------------------------------------------------------------
# dynamic span index vectors (Sec. 3.3.2): votes (Eq. 6), area ratios, Eq. 7
# ----------------------------------------------------------------------------
RATIO_ROW, RATIO_COL, RATIO_ROWCOL = 0, 1, 2


def token_votes(A: np.ndarray) -> np.ndarray:
    """Eq. 6: v_x = sum over heads and rows of A[., i, x]; A is the head-summed softmax map
    of the chunk (the rows of the chunk play the role of the window)."""
    return np.asarray(A, np.float64).sum(axis=0)


def span_area_ratio(A: np.ndarray, a: int, b: int, mode: int) -> float:
    """r_a of the span [a, b) (Sec. 3.3.2, the figure with Span1..Span4): area of the span's own
    triangle over that area plus its neighbours' -- the cells of the same rows left of the span
    (row), of the same columns below it (column), or both."""
    A = np.asarray(A, np.float64)
    tri = 0.0
    for i in range(a, b):
        tri += A[i, a:i + 1].sum()
    row = A[a:b, :a].sum()
    col = A[b:, a:b].sum()
    if mode == RATIO_ROW:
        den = tri + row
    elif mode == RATIO_COL:
        den = tri + col
    elif mode == RATIO_ROWCOL:
        den = tri + row + col
    else:
        raise ValueError(mode)
    return tri / den


def index_vector_count(length: int, r_a: float, lam: float, n_min: int, n_max: int) -> int:
    """Eq. 7 and the sentence after it: r_v = 1 / e^(lam (1 - r_a)); the span keeps
    round(length * r_v) index vectors (ties to even), clamped to [n_min, n_max] and to the
    span itself (at least one, at most its length)."""
    r_v = 1.0 / math.exp(lam * (1.0 - r_a))
    n = int(np.rint(length * r_v))
    n = max(n, n_min)
    if n_max > 0:
        n = min(n, n_max)
    return max(1, min(n, length))


def span_index_tokens(v: np.ndarray, a: int, b: int, count: int) -> np.ndarray:
    """The `count` tokens of [a, b) with the most votes (ties: the earlier token), ascending."""
    order = sorted(range(a, b), key=lambda t: (-v[t], t))
    return np.asarray(sorted(order[:count]), np.int64)


def share_block_budget(counts: Sequence[int], budget: int) -> List[int]:
    """The paper's cap of M index vectors per memory block (Sec. 4, "Compression Ratio": up to M span index
    vectors per block of 128 tokens), shared out over the block's spans. The paper does not say how; the
    reading taken here: if the spans' own counts (Eq. 7, clamped) add up to more than M, the largest counts
    are levelled down -- every span keeps min(count, level) for the highest level that fits, and what is left
    of M goes, one vector each, to the earliest spans still below their own count. Every span keeps at least
    one vector, so a block of more than M spans exceeds M by as many."""
    counts = [int(c) for c in counts]
    if budget <= 0 or sum(counts) <= budget:
        return counts
    level = 1
    while sum(min(c, level + 1) for c in counts) <= budget:
        level += 1
    out = [min(c, level) for c in counts]
    left = budget - sum(out)
    for i, c in enumerate(counts):
        if left <= 0:
            break
        if c > out[i]:
            out[i] += 1
            left -= 1
    return out


def dynamic_index_counts(A: np.ndarray, bounds: np.ndarray, lam: float, n_min: int, n_max: int, mode: int,
                         block_max: int = 0, unit: int = 0, c0: int = 0) -> List[int]:
    """Index vectors kept by every span of a chunk: Eq. 7 per span, then (block_max > 0) the budget of
    block_max vectors per memory block, a block being the part of a unit of `unit` tokens (absolute
    positions, the chunk starts at c0) that lies in this chunk; spans are cut at unit edges."""
    counts = []
    for s in range(len(bounds) - 1):
        a, b = int(bounds[s]), int(bounds[s + 1])
        counts.append(index_vector_count(b - a, span_area_ratio(A, a, b, mode), lam, n_min, n_max))
    if block_max > 0:
        if unit <= 0:
            raise ValueError("a budget per block needs memory units")
        blocks = {}
        for s in range(len(bounds) - 1):
            blocks.setdefault((c0 + int(bounds[s])) // unit, []).append(s)
        for members in blocks.values():
            shared = share_block_budget([counts[s] for s in members], block_max)
            for s, n in zip(members, shared):
                counts[s] = n
    return counts


def dynamic_index_tokens(A: np.ndarray, bounds: np.ndarray, lam: float, n_min: int, n_max: int,
                         mode: int, block_max: int = 0, unit: int = 0, c0: int = 0) -> List[np.ndarray]:
    """Index tokens (chunk-local, ascending) of every span of a chunk."""
    v = token_votes(A)
    counts = dynamic_index_counts(A, bounds, lam, n_min, n_max, mode, block_max, unit, c0)
    out = []
    for s in range(len(bounds) - 1):
        a, b = int(bounds[s]), int(bounds[s + 1])
        out.append(span_index_tokens(v, a, b, counts[s]))
    return out


def index_vector_sums(X: np.ndarray, tokens: Sequence[np.ndarray], dtype: str) -> np.ndarray:
    """One stored vector per span: the sum of the rows of X at its index tokens. Eq. 8 sums the
    dot products of all pairs of index vectors of two spans, which is the dot product of these
    sums. Rounded once to dtype."""
    X = np.asarray(X, np.float64)
    out = np.empty((len(tokens), X.shape[1]), np.float64)
    for s, t in enumerate(tokens):
        out[s] = X[t].sum(axis=0)
    return round_to_dtype(out, dtype)


def dynamic_index_is_stable(A: np.ndarray, bounds: np.ndarray, lam: float, n_min: int, n_max: int,
                            mode: int, rel: float = 2.0 ** -18, draws: int = 2, seed: int = 0,
                            block_max: int = 0, unit: int = 0, c0: int = 0) -> bool:
    """Audit: are the index tokens the same when every map cell moves by a relative `rel`?"""
    base = dynamic_index_tokens(A, bounds, lam, n_min, n_max, mode, block_max, unit, c0)
    rng = np.random.default_rng(seed)
    for _ in range(draws):
        p = rng.uniform(-rel, rel, size=A.shape)
        t = dynamic_index_tokens(A * (1.0 + p), bounds, lam, n_min, n_max, mode, block_max, unit, c0)
        if any(len(x) != len(y) or np.any(x != y) for x, y in zip(base, t)):
            return False
    return True


def span_scores(Qrep: np.ndarray, Krep: np.ndarray) -> np.ndarray:
    """score_i = max_j Qrep_j . Krep_i  (Eq. 8 with one vector per span, max over the
    query spans as in Eq. 9)."""
    sim = np.asarray(Qrep, np.float64) @ np.asarray(Krep, np.float64).T     # [n_q_spans, n_spans]
    return sim.max(axis=0)


def clipped_ranges(starts: np.ndarray, lens: np.ndarray, n_sink: int, win_start: int
                   ) -> Tuple[np.ndarray, np.ndarray]:
    """Part of every stored span that lies in the evicted region [n_sink, win_start)."""
    a = np.maximum(starts, n_sink)
    b = np.minimum(starts + lens, win_start)
    return a, b


def select_spans(scores: np.ndarray, clip_len: np.ndarray, eligible: np.ndarray,
                 k_max: int, budget_tokens: int) -> np.ndarray:
    """Top-K of Eq. 9 at span granularity: eligible spans by (-score, id); the longest
    prefix with sum(clipped length) <= budget (if > 0) and count <= k_max (if > 0).
    Returns the selected ids in ascending order."""
    ids = [int(i) for i in np.nonzero(eligible)[0]]
    ids.sort(key=lambda i: (-float(scores[i]), i))
    sel: List[int] = []
    total = 0
    for i in ids:
        if k_max and len(sel) >= k_max:
            break
        if budget_tokens and total + int(clip_len[i]) > budget_tokens:
            break
        sel.append(i)
        total += int(clip_len[i])
    return np.asarray(sorted(sel), dtype=np.int64)


def select_units(span_scores: np.ndarray, starts: np.ndarray, unit: int, n_tokens: int, n_sink: int,
                 win_start: int, k_max: int, budget_tokens: int) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 9 as written: the stream is cut into memory units (blocks) of `unit` tokens, a unit
    scores the maximum over its spans (a span belongs to the unit its first token lies in), and
    the top units are retrieved whole: units whose part in the evicted region [n_sink,
    win_start) is not empty, by (-score, id), the longest prefix with at most k_max units and at
    most budget_tokens evicted tokens. Returns (selected unit ids ascending, score of every unit)."""
    n_units = (n_tokens + unit - 1) // unit
    uscore = np.full(n_units, -np.inf)
    for s, a in zip(span_scores, starts):
        u = int(a) // unit
        uscore[u] = max(uscore[u], float(s))
    lo = np.maximum(np.arange(n_units) * unit, n_sink)
    hi = np.minimum(np.minimum((np.arange(n_units) + 1) * unit, n_tokens), win_start)
    sel = select_spans(uscore, hi - lo, lo < hi, k_max, budget_tokens)
    return sel, uscore


def collaborative_units(own_scores: np.ndarray, clip_len: np.ndarray, eligible: np.ndarray,
                        voters: Sequence[Tuple[float, Sequence[int]]], own_weight: float,
                        k_max: int, budget_tokens: int) -> Tuple[np.ndarray, np.ndarray]:
    """Sec. 3.5, Collaborative Voting, on memory units. `voters` = (weight, selected unit ids) of
    the preceding layers that take part, in layer order. The layer first selects on its own
    (Eq. 9); every voter and the layer itself then give their weight to each unit they selected;
    units are ordered by (-votes, -own score, id) and the longest prefix within k_max units and
    the token budget is the layer's selection. Votes are added in float32, voters first in
    their order, the layer last. Returns (selected unit ids ascending, votes)."""
    own = select_spans(own_scores, clip_len, eligible, k_max, budget_tokens)
    votes = np.zeros(len(own_scores), np.float32)
    for w, ids in voters:
        for u in ids:
            if u < len(votes):
                votes[u] = np.float32(votes[u] + np.float32(w))
    for u in own:
        votes[u] = np.float32(votes[u] + np.float32(own_weight))
    ids = [int(i) for i in np.nonzero(eligible)[0]]
    ids.sort(key=lambda i: (-float(votes[i]), -float(own_scores[i]), i))
    sel: List[int] = []
    total = 0
    for i in ids:
        if k_max and len(sel) >= k_max:
            break
        if budget_tokens and total + int(clip_len[i]) > budget_tokens:
            break
        sel.append(i)
        total += int(clip_len[i])
    return np.asarray(sorted(sel), dtype=np.int64), votes


# ----------------------------------------------------------------------------
# exact attention over an explicit key set (Sec. 3.4, third step)
# ----------------------------------------------------------------------------
def attend_rows(Q: np.ndarray, K: np.ndarray, V: np.ndarray, ctx_idx: np.ndarray,
                c0: int, rows: Optional[Sequence[int]] = None
                ) -> Tuple[np.ndarray, np.ndarray]:
    """softmax(q K^T / sqrt(d)) V for query rows of the chunk starting at c0.

    Q: [L, d] (one query head), K/V: [T, d] (its KV head), ctx_idx: token ids of the
    non-current part (initial | retrieved | window), shared by all rows; row i also
    sees the current tokens c0..c0+i.  Returns (O [len(rows), d], lse [len(rows)]).
    """
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    L, d = Q.shape
    rows = list(range(L)) if rows is None else list(rows)
    Kc, Vc = K[ctx_idx], V[ctx_idx]
    zc = (Q[rows] @ Kc.T) / math.sqrt(d)                   # [r, n_ctx]
    O = np.empty((len(rows), d))
    lse = np.empty(len(rows))
    for r, i in enumerate(rows):
        zl = (K[c0:c0 + i + 1] @ Q[i]) / math.sqrt(d)
        z = np.concatenate([zc[r], zl])
        m = z.max()
        p = np.exp(z - m)
        den = p.sum()
        O[r] = (p[:len(ctx_idx)] @ Vc + p[len(ctx_idx):] @ V[c0:c0 + i + 1]) / den
        lse[r] = m + math.log(den)
    return O, lse


# ----------------------------------------------------------------------------
# the streaming step for one (layer, sequence): all KV heads
# ----------------------------------------------------------------------------
@dataclass
class OracleConfig:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                 # "f32" | "bf16": dtype the representative vectors are stored in
    n_sink: int
    window: int
    k_max: int = 0
    budget_tokens: int = 0
    seg_map: int = MAP_LOGIT
    theta: float = 0.0
    phi: float = 0.0
    max_spans_per_chunk: int = 0
    theta_quantile: float = 0.0   # > 0: theta is this percentile of the chunk's map (theta is ignored)
    unit_tokens: int = 0          # > 0: retrieval by memory units of this many tokens (Eq. 9), spans cut at their edges
    rep_mode: int = 0          # REP_MEAN | REP_DYNAMIC
    lam: float = 3.0           # lambda of Eq. 7
    n_min: int = 1             # fewest / most index vectors per span (0 = no upper limit)
    n_max: int = 0
    ratio_mode: int = RATIO_ROW
    block_max: int = 0         # > 0: at most this many index vectors per memory block (the paper's M), needs unit_tokens

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


class OracleStream:
    """Index memory + the three steps for one sequence of one layer.

    K, V: [Hkv][T][d] full streams (only tokens already appended are read),
    held by reference."""

    def __init__(self, cfg: OracleConfig, K: np.ndarray, V: np.ndarray):
        self.cfg = cfg
        self.K = np.asarray(K, np.float64)
        self.V = np.asarray(V, np.float64)
        H = cfg.n_kv_heads
        self.n_tokens = 0
        self.starts: List[List[int]] = [[] for _ in range(H)]
        self.lens: List[List[int]] = [[] for _ in range(H)]
        self.krep: List[List[np.ndarray]] = [[] for _ in range(H)]
        self.last_chunk: Tuple[int, int] = (0, 0)                  # (c0, L)
        self.last_bounds: List[np.ndarray] = [np.zeros(0, np.int64) for _ in range(H)]
        self.last_index_tokens: List[List[np.ndarray]] = [[] for _ in range(H)]   # REP_DYNAMIC only
        self.sel: List[np.ndarray] = [np.zeros(0, np.int64) for _ in range(H)]
        self.sel_scores: List[np.ndarray] = [np.zeros(0) for _ in range(H)]

    # -- step 1 -------------------------------------------------------------
    def append_chunk(self, n_new: int, q_seg: Optional[np.ndarray] = None,
                     bounds: Optional[Sequence[np.ndarray]] = None) -> None:
        """Segment tokens [T, T+n_new), store spans and representative keys.

        q_seg: [n_new][Hq][d] queries used to build the map, or None (keys are used).
        bounds: per KV head chunk-local boundaries to use instead of segmenting."""
        c = self.cfg
        c0 = self.n_tokens
        for h in range(c.n_kv_heads):
            Kc = self.K[h, c0:c0 + n_new]
            if bounds is not None:
                b = np.asarray(bounds[h], np.int64)
            else:
                Qg = None
                if q_seg is not None:
                    Qg = np.asarray(q_seg, np.float64)[:, h * c.group:(h + 1) * c.group, :]
                    Qg = np.transpose(Qg, (1, 0, 2))
                b = segment_chunk(Kc, Qg, c.seg_map, c.theta, c.phi, c.max_spans_per_chunk,
                                  theta_quantile=c.theta_quantile, unit=c.unit_tokens, c0=c0)
            if c.rep_mode == REP_DYNAMIC:
                Qg = None
                if q_seg is not None:
                    Qg = np.transpose(np.asarray(q_seg, np.float64)[:, h * c.group:(h + 1) * c.group, :], (1, 0, 2))
                A, _ = chunk_map(Kc, Qg, MAP_SOFTMAX)            # votes and areas come from the softmax map
                toks = dynamic_index_tokens(A, b, c.lam, c.n_min, c.n_max, c.ratio_mode, c.block_max,
                                            c.unit_tokens, c0)
                self.last_index_tokens[h] = toks
                reps = index_vector_sums(Kc, toks, c.dtype)
            else:
                reps = span_means(Kc, b, c.dtype)
            for s in range(len(b) - 1):
                self.starts[h].append(c0 + int(b[s]))
                self.lens[h].append(int(b[s + 1] - b[s]))
                self.krep[h].append(reps[s])
            self.last_bounds[h] = b
        self.last_chunk = (c0, n_new)
        self.n_tokens = c0 + n_new

    def win_start(self, c0: int) -> int:
        return max(min(self.cfg.n_sink, c0), c0 - self.cfg.window)

    # -- step 2 -------------------------------------------------------------
    def retrieve(self, q: np.ndarray) -> List[np.ndarray]:
        """q: [L][Hq][d] queries of the last appended chunk.  Selected span ids per KV head."""
        c = self.cfg
        c0, L = self.last_chunk
        q = np.asarray(q, np.float64)
        assert q.shape[0] == L
        ws = self.win_start(c0)
        out = []
        for h in range(c.n_kv_heads):
            qsum = q[:, h * c.group:(h + 1) * c.group, :].sum(axis=1)        # sum over the group's heads
            if c.rep_mode == REP_DYNAMIC:
                Qrep = index_vector_sums(qsum, self.last_index_tokens[h], c.dtype)
            else:
                Qrep = span_means(qsum, self.last_bounds[h], c.dtype)
            starts = np.asarray(self.starts[h], np.int64)
            lens = np.asarray(self.lens[h], np.int64)
            a, b = clipped_ranges(starts, lens, min(c.n_sink, c0), ws)
            eligible = a < b
            scores = span_scores(Qrep, np.stack(self.krep[h]))
            if c.unit_tokens > 0:
                sel, _ = select_units(scores, starts, c.unit_tokens, c0 + L, min(c.n_sink, c0), ws, c.k_max,
                                      c.budget_tokens)
            else:
                sel = select_spans(scores, b - a, eligible, c.k_max, c.budget_tokens)
            self.sel[h] = sel
            self.sel_scores[h] = scores
            out.append(sel)
        return out

    def retrieve_collaborative(self, q: np.ndarray, preceding: Sequence["OracleStream"],
                               weights: Sequence[float], own_weight: float) -> List[np.ndarray]:
        """Step 2 with the votes of the preceding layers (Sec. 3.5, Collaborative Voting); needs
        retrieval by memory units. preceding[k] is the stream of an earlier layer of the same
        sequence (its current selection votes with weights[k]; weight 0 = takes no part)."""
        c = self.cfg
        assert c.unit_tokens > 0
        c0, L = self.last_chunk
        q = np.asarray(q, np.float64)
        ws = self.win_start(c0)
        U = c.unit_tokens
        n_units = (c0 + L + U - 1) // U
        out = []
        for h in range(c.n_kv_heads):
            qsum = q[:, h * c.group:(h + 1) * c.group, :].sum(axis=1)
            if c.rep_mode == REP_DYNAMIC:
                Qrep = index_vector_sums(qsum, self.last_index_tokens[h], c.dtype)
            else:
                Qrep = span_means(qsum, self.last_bounds[h], c.dtype)
            scores = span_scores(Qrep, np.stack(self.krep[h]))
            uscore = np.full(n_units, -np.inf)
            for sc_, a in zip(scores, self.starts[h]):
                uscore[a // U] = max(uscore[a // U], float(sc_))
            lo = np.maximum(np.arange(n_units) * U, min(c.n_sink, c0))
            hi = np.minimum(np.minimum((np.arange(n_units) + 1) * U, c0 + L), ws)
            voters = [(w, [int(u) for u in p.sel[h]]) for p, w in zip(preceding, weights) if w > 0]
            sel, _ = collaborative_units(uscore, hi - lo, lo < hi, voters, own_weight, c.k_max, c.budget_tokens)
            self.sel[h] = sel
            self.sel_scores[h] = scores
            out.append(sel)
        return out

    def force_selection(self, h: int, ids: Sequence[int]) -> None:
        self.sel[h] = np.asarray(sorted(int(i) for i in ids), np.int64)

    def retrieve_persistent(self) -> List[np.ndarray]:
        """Sec. 3.5, Persistent Mechanism: no scoring; the spans selected earlier (for the last
        prefill chunk) stay selected for the chunk appended last. The context set follows from
        them and from where the window is now (context_tokens)."""
        return [s.copy() for s in self.sel]

    # -- step 3 -------------------------------------------------------------
    def context_tokens(self, h: int) -> np.ndarray:
        """Token ids of initial | retrieved (clipped) | window for the last chunk, ascending."""
        c = self.cfg
        c0, _ = self.last_chunk
        n_sink = min(c.n_sink, c0)
        ws = self.win_start(c0)
        parts = [np.arange(0, n_sink)]
        for i in self.sel[h]:
            if c.unit_tokens > 0:                          # the selection holds unit ids
                a = max(int(i) * c.unit_tokens, n_sink)
                b = min((int(i) + 1) * c.unit_tokens, ws)
            else:
                a = max(self.starts[h][i], n_sink)
                b = min(self.starts[h][i] + self.lens[h][i], ws)
            if a < b:
                parts.append(np.arange(a, b))
        parts.append(np.arange(ws, c0))
        return np.concatenate(parts).astype(np.int64)

    def attend(self, q: np.ndarray, rows: Optional[Sequence[int]] = None,
               heads: Optional[Sequence[int]] = None) -> Tuple[np.ndarray, np.ndarray]:
        """q: [L][Hq][d].  Returns O [len(rows)][len(heads)][d], lse [len(rows)][len(heads)]."""
        c = self.cfg
        c0, L = self.last_chunk
        q = np.asarray(q, np.float64)
        rows = list(range(L)) if rows is None else list(rows)
        heads = list(range(c.n_q_heads)) if heads is None else list(heads)
        O = np.empty((len(rows), len(heads), c.head_dim))
        lse = np.empty((len(rows), len(heads)))
        ctx_cache = {}
        for k, g in enumerate(heads):
            h = g // c.group
            if h not in ctx_cache:
                ctx_cache[h] = self.context_tokens(h)
            o, l = attend_rows(q[:, g, :], self.K[h], self.V[h], ctx_cache[h], c0, rows)
            O[:, k, :] = o
            lse[:, k] = l
        return O, lse


def full_causal_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, pos: Sequence[int]
                          ) -> np.ndarray:
    """Textbook causal softmax attention for query positions `pos` (one head):
    row t attends keys 0..t.  Q: [T, d] indexed by absolute position."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    d = Q.shape[1]
    out = np.empty((len(pos), d))
    for r, t in enumerate(pos):
        z = (K[:t + 1] @ Q[t]) / math.sqrt(d)
        p = np.exp(z - z.max())
        out[r] = (p @ V[:t + 1]) / p.sum()
    return out
