"""CPU oracle for METok's token-compression path (arXiv 2506.02850).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke check
and the bench's ``cpu_baseline`` leg may import this module.  It shares no code
with the HIP library and never calls it; the HIP library never calls this.

Everything is the paper's definition written out in numpy float64, one step per
function, in the paper's order and notation, with no blocking, fusion or
reordering.  METok is a heuristic pipeline, so the oracle is "the algorithm
step by step", computed in double precision from the same (already rounded)
input values the GPU sees.

Where the paper is silent or inconsistent the reading taken is named next to
the function.  Readings that nothing in the paper can confirm are marked
"parity unpinned": Eq. 4 as a Frobenius cosine of the flattened frames, Eq. 5
as a per-token cosine averaged over the frame, the text-to-visual attention
score as the head- and query-mean of causal softmax probabilities, and the
per-class (rather than per-event) retention quota.  The arithmetic of each of
those functions is still pinned by brute force, closed forms and invariants in
the CPU tests; it is the *choice of formula* that is unpinned.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64
ZERO_NORM = 1e-12          # a cosine whose denominator is below this is defined as 0
CEIL_SLACK = 1e-9          # ceil(x - 1e-9): keeps 0.55 * 20 = 11.000000000000002 at 11

EVENT_REDUCE_MEAN = 0      # Sec. 3.2.1: the event score is the mean of its frames' scores
EVENT_REDUCE_MAX = 1       # Algorithm 1: r_j = max over the event's frames
SIM_FLAT = 0               # Eq. 4 over all N*d entries of the two frames
SIM_TOKEN_MEAN = 1         # mean over the N token positions of the cosine of matching tokens
SIM_POOLED = 2             # cosine of the two frames' token-mean vectors
SCORE_CAUSAL_ALL = 0       # softmax over every key a text query can see
SCORE_VISUAL_ONLY = 1      # softmax over the visual keys only
POOL_FLOOR = 0             # trailing cells that do not fill a window are dropped
POOL_CEIL = 1              # partial edge windows are averaged over their valid cells


def ceil_ratio(x: float) -> int:
    """The only rounding the paper states is the ceiling in ceil(alpha k) (Sec. 3.2.1);
    every ratio-to-count conversion uses the same rule, guarded against binary noise."""
    return int(math.ceil(float(x) - CEIL_SLACK))


def _cos(num: float, den: float) -> float:
    return 0.0 if den < ZERO_NORM else num / den


# ---------------------------------------------------------------------------
# Stage 1 (Sec. 3.2.1, Algorithm 1)
# ---------------------------------------------------------------------------
def adjacent_frame_cosine(V: np.ndarray, mode: int = SIM_FLAT) -> np.ndarray:
    """Eq. 4: S_i = <v_i, v_{i+1}> / (||v_i|| ||v_{i+1}||) for the T-1 adjacent pairs.

    v_i is the whole N x d frame.  SIM_FLAT (default reading): the inner product and the norms run
    over all N*d entries (Frobenius).  The other two readings of "cosine of two N x d embeddings":
    SIM_TOKEN_MEAN averages the cosines of the N matching token pairs, SIM_POOLED takes the cosine of
    the frames' mean tokens.  Index i = 0..T-2 pairs frame i with i+1.
    """
    V = np.asarray(V, dtype=F64)
    T, N, _ = V.shape
    S = np.zeros(max(T - 1, 0), dtype=F64)
    for i in range(T - 1):
        if mode == SIM_FLAT:
            a = V[i].reshape(-1)
            b = V[i + 1].reshape(-1)
            S[i] = _cos(float(np.dot(a, b)), math.sqrt(float(np.dot(a, a))) * math.sqrt(float(np.dot(b, b))))
        elif mode == SIM_TOKEN_MEAN:
            acc = 0.0
            for n in range(N):
                a, b = V[i, n], V[i + 1, n]
                acc += _cos(float(np.dot(a, b)), math.sqrt(float(np.dot(a, a))) * math.sqrt(float(np.dot(b, b))))
            S[i] = acc / N
        elif mode == SIM_POOLED:
            a = V[i].sum(axis=0) / N
            b = V[i + 1].sum(axis=0) / N
            S[i] = _cos(float(np.dot(a, b)), math.sqrt(float(np.dot(a, a))) * math.sqrt(float(np.dot(b, b))))
        else:
            raise ValueError("unknown similarity mode")
    return S


def event_boundaries(S: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Sec. 3.2.1: the k-1 lowest S_i are the boundaries; they split T frames into k events.

    A boundary at i means frame i+1 opens a new event.  Equal similarities are
    taken lowest index first.  Returns (event_start[k+1], frame_event[T]).
    """
    S = np.asarray(S, dtype=F64)
    T = S.shape[0] + 1
    if not (1 <= k <= T):
        raise ValueError("need 1 <= k <= T")
    order = sorted(range(T - 1), key=lambda i: (S[i], i))
    cuts = sorted(order[: k - 1])
    event_start = np.array([0] + [c + 1 for c in cuts] + [T], dtype=np.int32)
    frame_event = np.zeros(T, dtype=np.int32)
    for e in range(k):
        frame_event[event_start[e]: event_start[e + 1]] = e
    return event_start, frame_event


def frame_text_score(V: np.ndarray, t: np.ndarray) -> np.ndarray:
    """Eq. 5: cosine between a frame's visual embeddings and the text embedding t.

    Reading: the cosine is taken per token (row of v_i) and averaged over the
    frame's N tokens, giving one score per frame.
    """
    V = np.asarray(V, dtype=F64)
    t = np.asarray(t, dtype=F64).reshape(-1)
    T, N, _ = V.shape
    tn = math.sqrt(float(np.dot(t, t)))
    f = np.zeros(T, dtype=F64)
    for i in range(T):
        acc = 0.0
        for n in range(N):
            row = V[i, n]
            acc += _cos(float(np.dot(row, t)), math.sqrt(float(np.dot(row, row))) * tn)
        f[i] = acc / N
    return f


def key_events_and_frames(f: np.ndarray, event_start: np.ndarray, alpha: float, beta: float,
                          event_reduce: int = EVENT_REDUCE_MEAN):
    """Sec. 3.2.1: event score = average of its frames' text scores (Algorithm 1
    prints max instead; selectable); the ceil(alpha k) best events are key; in
    every event the top-beta share of frames, ceil(beta |E_j|), are key frames.
    Ties go to the lower index.  Returns (event_score, event_is_key, frame_is_key).
    """
    f = np.asarray(f, dtype=F64)
    k = len(event_start) - 1
    score = np.zeros(k, dtype=F64)
    for j in range(k):
        seg = f[event_start[j]: event_start[j + 1]]
        score[j] = float(seg.mean()) if event_reduce == EVENT_REDUCE_MEAN else float(seg.max())
    n_key = min(k, ceil_ratio(alpha * k))
    event_is_key = np.zeros(k, dtype=np.uint8)
    for j in sorted(range(k), key=lambda j: (-score[j], j))[:n_key]:
        event_is_key[j] = 1
    frame_is_key = np.zeros(f.shape[0], dtype=np.uint8)
    for j in range(k):
        frames = list(range(int(event_start[j]), int(event_start[j + 1])))
        n_kf = min(len(frames), ceil_ratio(beta * len(frames)))
        for i in sorted(frames, key=lambda i: (-f[i], i))[:n_kf]:
            frame_is_key[i] = 1
    return score, event_is_key, frame_is_key


def pooling_strides(event_start: np.ndarray, event_is_key: np.ndarray, frame_is_key: np.ndarray,
                    alpha: float, s1: int, s2: int, grid: Tuple[int, int]) -> np.ndarray:
    """Sec. 3.2.1 "Adaptive Pooling Strategy" / Algorithm 1: stride s1 for key frames and s2
    for non-key frames of key events; both scaled by 1/alpha in non-key events.
    A non-integer s/alpha is rounded up (the scaling is there to pool non-key
    events harder); strides are clamped to [1, max(grid)]."""
    T = int(event_start[-1])
    g = max(grid)
    out = np.zeros(T, dtype=np.int32)
    for j in range(len(event_start) - 1):
        for i in range(int(event_start[j]), int(event_start[j + 1])):
            s = s1 if frame_is_key[i] else s2
            if not event_is_key[j]:
                s = ceil_ratio(s / alpha)
            out[i] = min(max(int(s), 1), g)
    return out


def pooled_side(g: int, s: int, edge: int) -> int:
    return max(1, g // s) if edge == POOL_FLOOR else -(-g // s)


def pool_frame(v: np.ndarray, grid: Tuple[int, int], s: int, edge: int = POOL_FLOOR) -> np.ndarray:
    """pool2d(v_i, s) of Algorithm 1: non-overlapping s x s average over the frame's
    token grid (tokens are row-major over grid_h x grid_w), per channel.

    edge == POOL_FLOOR: output side floor(g/s), trailing cells that do not fill a
    window are dropped.  This is what the paper's own numbers imply: its base
    LLaVA-OneVision-7B KV cache (Table 3) corresponds to 13 x 13 = 169 tokens per
    27 x 27 frame under uniform stride 2, not 14 x 14.
    edge == POOL_CEIL: output side ceil(g/s), edge windows average their valid cells.
    """
    gh, gw = grid
    v = np.asarray(v, dtype=F64).reshape(gh, gw, -1)
    oh, ow = pooled_side(gh, s, edge), pooled_side(gw, s, edge)
    out = np.zeros((oh * ow, v.shape[2]), dtype=F64)
    for oy in range(oh):
        for ox in range(ow):
            win = v[oy * s: min((oy + 1) * s, gh), ox * s: min((ox + 1) * s, gw), :]
            out[oy * ow + ox] = win.reshape(-1, v.shape[2]).sum(axis=0) / (win.shape[0] * win.shape[1])
    return out


def compress_encoder_tokens(V: np.ndarray, grid: Tuple[int, int], t: np.ndarray, event_start: np.ndarray,
                            alpha: float, beta: float, s1: int, s2: int,
                            event_reduce: int = EVENT_REDUCE_MEAN, edge: int = POOL_FLOOR,
                            frame_score: Optional[np.ndarray] = None):
    """Algorithm 1 after segmentation: score frames, pick key events/frames, pool every
    frame with its stride and append the pooled frames in temporal order.

    Returns a dict with tokens [M, d] (float64), frame_offsets [T+1], token_event [M],
    event_is_key, frame_is_key, frame_stride, frame_score, event_score.
    """
    V = np.asarray(V, dtype=F64)
    T = V.shape[0]
    f = frame_text_score(V, t) if frame_score is None else np.asarray(frame_score, dtype=F64)
    ev_score, ev_key, fr_key = key_events_and_frames(f, event_start, alpha, beta, event_reduce)
    stride = pooling_strides(event_start, ev_key, fr_key, alpha, s1, s2, grid)
    pieces: List[np.ndarray] = []
    offsets = np.zeros(T + 1, dtype=np.int32)
    token_event: List[int] = []
    for j in range(len(event_start) - 1):
        for i in range(int(event_start[j]), int(event_start[j + 1])):
            p = pool_frame(V[i], grid, int(stride[i]), edge)
            pieces.append(p)
            offsets[i + 1] = offsets[i] + p.shape[0]
            token_event.extend([j] * p.shape[0])
    tokens = np.concatenate(pieces, axis=0) if pieces else np.zeros((0, V.shape[2]), dtype=F64)
    return dict(tokens=tokens, frame_offsets=offsets, token_event=np.asarray(token_event, dtype=np.int32),
                event_is_key=ev_key, frame_is_key=fr_key, frame_stride=stride, frame_score=f,
                event_score=ev_score)


# ---------------------------------------------------------------------------
# Stage 2 (Sec. 3.2.2, Eq. 6-7)
# ---------------------------------------------------------------------------
def text_to_visual_attention(q_text: np.ndarray, k_all: np.ndarray, vis_start: int, n_vis: int,
                             mode: int = SCORE_CAUSAL_ALL) -> np.ndarray:
    """Sec. 3.2.2 "visual-text attention scores" (the paper gives no formula).

    Reading: q_text [Hq, Tq, dh] are the queries of the last Tq sequence
    positions (the text), k_all [Hkv, S, dh] the keys of the whole sequence;
    query head h reads kv head h // (Hq / Hkv).  Each query at position p runs
    an ordinary causal softmax over keys 0..p of q.k / sqrt(dh); a_j is the
    probability that lands on visual key j, averaged over all heads and queries.
    SCORE_VISUAL_ONLY normalises over the visual keys alone (prefix and text keys
    take no probability mass).
    """
    q = np.asarray(q_text, dtype=F64)
    k = np.asarray(k_all, dtype=F64)
    Hq, Tq, dh = q.shape
    Hkv, S, _ = k.shape
    group = Hq // Hkv
    a = np.zeros(n_vis, dtype=F64)
    pos = np.arange(S)
    for h in range(Hq):
        logits = (q[h] @ k[h // group].T) / math.sqrt(dh)          # [Tq, S]
        for i in range(Tq):
            p_i = S - Tq + i
            visible = pos <= p_i
            if mode == SCORE_VISUAL_ONLY:
                visible = visible & (pos >= vis_start) & (pos < vis_start + n_vis)
            row = np.where(visible, logits[i], -np.inf)
            row = np.exp(row - row.max())
            row = row / row.sum()
            a += row[vis_start: vis_start + n_vis]
    return a / (Hq * Tq)


def event_weighted_scores(a: np.ndarray, token_event: np.ndarray, event_weight: Optional[np.ndarray]) -> np.ndarray:
    """score_j = w_{e(j)} a_j: attention alignment modulated by the importance of the token's event."""
    a = np.asarray(a, dtype=F64)
    if event_weight is None:
        return a.copy()
    return a * np.asarray(event_weight, dtype=F64)[np.asarray(token_event)]


def retention_ratios(level: int, r: float, alpha: float) -> Tuple[float, float]:
    """Eq. 6-7 at the layer boundaries l_1, l_2, l_3 (level = 1, 2, 3; 0 = before l_1).

    R_key: 1, r, r^2, 0.  R_non-key: 1, alpha r, 0, 0.  The printed cases leave
    l = l_3 (and l = l_2 for non-key) undefined; they are read as >=.
    """
    key = [1.0, r, r * r, 0.0][level]
    non = [1.0, alpha * r, 0.0, 0.0][level]
    return key, non


def retention_quotas(level: int, r: float, alpha: float, n_key_orig: int, n_non_orig: int) -> Tuple[int, int]:
    """Token counts for Eq. 6-7: ratios are relative to the tokens originally passed to the LLM."""
    rk, rn = retention_ratios(level, r, alpha)
    return min(n_key_orig, ceil_ratio(rk * n_key_orig)), min(n_non_orig, ceil_ratio(rn * n_non_orig))


def segmented_topk(scores: np.ndarray, token_seg: np.ndarray, seg_quota: Sequence[int]) -> np.ndarray:
    """Sec. 3.2.2: in every segment keep the quota best-scored tokens (ties: lower index first).
    Returns the kept positions in ascending order (temporal order is preserved)."""
    scores = np.asarray(scores)
    token_seg = np.asarray(token_seg)
    kept: List[int] = []
    for s, quota in enumerate(seg_quota):
        members = [j for j in range(scores.shape[0]) if token_seg[j] == s]
        if quota > len(members):
            raise ValueError("quota exceeds segment population")
        kept.extend(sorted(members, key=lambda j: (-scores[j], j))[: int(quota)])
    return np.asarray(sorted(kept), dtype=np.int32)


def compact_hidden(hidden: np.ndarray, vis_start: int, n_vis: int, kept: np.ndarray) -> np.ndarray:
    """Rows of X = [prefix; X_vis; X_text] after pruning: prefix, kept visual rows in order, text."""
    hidden = np.asarray(hidden)
    return np.concatenate([hidden[:vis_start], hidden[vis_start + np.asarray(kept, dtype=np.int64)],
                           hidden[vis_start + n_vis:]], axis=0)


def prefill_prune(hidden, q_text, k_all, vis_start, n_vis, token_seg, token_event, event_weight,
                  seg_quota, orig_idx=None, scores=None):
    """One pruning layer: score, select per segment, compact hidden states and carried metadata."""
    if scores is None:
        a = text_to_visual_attention(q_text, k_all, vis_start, n_vis)
        scores = event_weighted_scores(a, token_event, event_weight)
    kept = segmented_topk(scores, token_seg, seg_quota)
    if orig_idx is None:
        orig_idx = np.arange(n_vis, dtype=np.int32)
    return dict(scores=np.asarray(scores, dtype=F64), kept_idx=kept,
                hidden_out=compact_hidden(hidden, vis_start, n_vis, kept),
                token_seg_out=np.asarray(token_seg)[kept], token_event_out=np.asarray(token_event)[kept],
                orig_idx_out=np.asarray(orig_idx)[kept])


# ---------------------------------------------------------------------------
# Stage 3 (Sec. 3.3)
# ---------------------------------------------------------------------------
def kv_compact(slab: np.ndarray, idx: Optional[np.ndarray]) -> np.ndarray:
    """Row i of the compacted [S, dh] slab is row idx[i] of the old one (None = keep all)."""
    slab = np.asarray(slab)
    return slab.copy() if idx is None else slab[np.asarray(idx, dtype=np.int64)]


def kv_relink_pages(idx: np.ndarray, len_in: int, page_size: int, table_in: Sequence[int]) -> dict:
    """Sec. 3.3 on a paged cache, as a pure index transformation (no rows are touched here).

    The compacted sequence keeps the old logical rows idx[0] < idx[1] < ... as its rows 0, 1, ...; its
    pages are described by a new page table over the physical pages the sequence already owns:
      * a new page whose rows are exactly one whole old page (in order, from that page's first slot) is
        "relinked": it takes over that old page's physical page and none of its rows is copied;
      * the old pages not taken over in this way are free; the new pages that are not relinked take them
        in ascending order (k-th such new page -> k-th free old page) and are filled by row copies;
      * the free old pages that are left are released.
    Returns table_out (physical page of every new page), free_pages (released physical pages, in
    ascending old-page order), relinked (flag per new page), home (old logical page whose physical page
    each new page occupies) and rows_copied (rows whose physical place changes).
    """
    idx = [int(x) for x in idx]
    n = len(idx)
    ps = int(page_size)
    n_old = -(-int(len_in) // ps)
    n_new = -(-n // ps)
    relinked, home, taken = [], [], set()
    for D in range(n_new):
        rows = idx[D * ps: min((D + 1) * ps, n)]
        whole = rows[0] % ps == 0 and rows == list(range(rows[0], rows[0] + len(rows))) and rows[0] + len(rows) <= len_in
        relinked.append(bool(whole))
        home.append(rows[0] // ps if whole else None)
        if whole:
            taken.add(rows[0] // ps)
    free_old = [j for j in range(n_old) if j not in taken]
    k = 0
    for D in range(n_new):
        if not relinked[D]:
            home[D] = free_old[k]
            k += 1
    table_out = [int(table_in[h]) for h in home]
    free_pages = [int(table_in[j]) for j in free_old[k:]]
    rows_copied = sum(1 for d in range(n) if home[d // ps] * ps + d % ps != idx[d])
    return dict(table_out=table_out, free_pages=free_pages, relinked=relinked, home=home, rows_copied=rows_copied)


def kv_text_only_schedule(n_layers: int, l1: int, n_vis: int, n_text: int) -> List[Optional[np.ndarray]]:
    """Sec. 3.3: layers below l_1 cache visual and text tokens; from l_1 on every visual
    token leaves the cache.  Layers are numbered from 0."""
    text = np.arange(n_vis, n_vis + n_text, dtype=np.int32)
    return [None if l < l1 else text for l in range(n_layers)]


def kv_token_layers(n_layers: int, l1: int, n_vis: int, n_text: int) -> int:
    """Cached (token, layer) pairs under the Sec. 3.3 rule; times bytes per token-layer = KV size."""
    return l1 * (n_vis + n_text) + (n_layers - l1) * n_text


def account(event_len: Sequence[int], event_is_key: Sequence[int], grid: Tuple[int, int], alpha: float, beta: float,
            s1: int, s2: int, pool_edge: int, r: float, L_H: Sequence[int], n_layers: int, n_text: int) -> dict:
    """Token and cache bookkeeping of the three stages in closed form (no tensors).

    Stage 1 (Sec. 3.2.1): event j of length n has ceil(beta n) key frames; a frame pooled with stride s
    leaves side(gh, s) * side(gw, s) tokens.  Stage 2 (Eq. 6-7): from layer l_i on, the key / non-key
    populations shrink to the level-i quotas of the counts that entered the LLM.  Stage 3 (Sec. 3.3):
    layers below l_1 cache everything they saw, the others the text rows only.
    Counts are tokens or (token, layer) pairs; multiply the latter by the bytes of one token in one layer.
    """
    gh, gw = grid
    g = max(grid)

    def rows(s: float) -> int:
        s = min(max(int(ceil_ratio(s)), 1), g)
        return pooled_side(gh, s, pool_edge) * pooled_side(gw, s, pool_edge)

    key = non = 0
    for n, is_key in zip(event_len, event_is_key):
        n = int(n)
        n_kf = min(n, ceil_ratio(beta * n))
        if is_key:
            key += n_kf * rows(s1) + (n - n_kf) * rows(s2)
        else:
            non += n_kf * rows(s1 / alpha) + (n - n_kf) * rows(s2 / alpha)
    level_tokens = [key + non] + [sum(retention_quotas(i, r, alpha, key, non)) for i in (1, 2, 3)]
    prefill = 0
    for l in range(n_layers):
        level = sum(1 for b in L_H if l >= b)
        prefill += level_tokens[level] + n_text
    return dict(tokens_encoder=int(sum(int(n) for n in event_len)) * gh * gw, tokens_llm=key + non, tokens_key=key,
                tokens_non=non, level_tokens=level_tokens, prefill_token_layers=prefill,
                kv_token_layers_full=n_layers * (key + non + n_text),
                kv_token_layers_stage2=prefill,
                kv_token_layers_stage3=kv_token_layers(n_layers, min(int(L_H[0]), n_layers), key + non, n_text))


# ---------------------------------------------------------------------------
# output rounding used when a merged feature is stored in bf16
# ---------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float64 -> nearest-even bf16 value, returned as float64 (finite inputs)."""
    x = np.asarray(x, dtype=F64)
    m, e = np.frexp(x)                       # x = m 2^e, 0.5 <= |m| < 1; bf16 keeps 8 significant bits
    return np.ldexp(np.rint(m * 256.0), e - 8)
