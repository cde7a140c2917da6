"""CPU oracle for the MoE-layer forward.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 statement of what one Mixture-of-Experts layer computes, written from
the paper (HarMoEny, arXiv 2506.12417) and the textbook definitions it relies on.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may call it; the product (the HIP
library and its Python binding) never does, and this file shares no code with it.

What follows which passage:

  route_topk        section 2, "Mixture-of-Experts": the router gives every expert a value in
                    (0,1) and the token goes to the k highest; Alg. 1 step 1 (m_expert).
  permute           Alg. 1 step 4 and the initial schedule S_initial of step 3, collapsed to one
                    GPU: tokens are grouped by their target expert (counts = the G=1 slice of
                    S_initial).
  expert_ffn        section 2 (two dense layers with an activation between) and section 4.4
                    (the expert is x W1 W2 with W1: m x p, W2: p x m; no biases).
  moe_layer         Alg. 1 steps 5-6 read as the result they must produce: each token's output is
                    the gate-weighted sum of its k experts' FFN outputs, in the original token
                    order (step 6, "reconstruct").  Computed per token straight from the
                    definition, without the permutation, so a permutation mistake cannot cancel.
  combine           Alg. 1 step 6 on already-permuted expert outputs.
  rebalance         Alg. 2 / section 4.2 (token rebalancing): pick_move() takes one decision of
                    the greedy loop, rebalance() applies decisions until none is left.
  token_threshold_q section 4.4, Eq. 1-4 and appendix B.
  schedule_*        the schedules a plan is made from: Alg. 2 with bins for GPUs (harmoeny), its
                    starting placement (static), section 5.3.2's round-robin placement and
                    even split.
  schedule_balanced, block_order, tiles_from_schedule
                    PARITY UNPINNED to the paper: the tile-equalising variant of Alg. 2 and the
                    order in which a bin lists its work are this library's own choices (the paper
                    leaves the order inside a GPU open).  They are pinned to Alg. 2 where they
                    coincide with it, to hand-worked cases and to invariants only.

Readings where the paper is silent (each listed in the design notes): the gate is a softmax over
all E logits; selection is on the logits, descending, ties to the lower expert index; with
renorm=1 the k gate values are divided by their sum; rows of one expert keep ascending
assignment order (assignment id a = t*k + j); expert FFNs have no bias.

bf16 tensors arrive as uint16 bit patterns and are widened exactly to float64; nothing is
rounded on the way except where a function says so.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence, Tuple

from fractions import Fraction

import numpy as np


# ----------------------------------------------------------------------------- number formats
def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening: uint16 is read as bfloat16 bits, float32/float64 as they are."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float64 -> nearest bfloat16 value (ties to even), returned as float64.  Only used by the
    diagnostic mode of expert_ffn; not part of the layer's definition."""
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- step 1: routing
def router_logits(x: np.ndarray, W_g: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    """l[t,e] = b[e] + sum_i x[t,i] W_g[i,e], float64."""
    l = to_f64(x) @ to_f64(W_g)
    if b is not None:
        l = l + to_f64(b)[None, :]
    return l


def route_topk(x: np.ndarray, W_g: np.ndarray, b: Optional[np.ndarray], k: int, renorm: int
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Top-k gating (section 2).  Returns (expert_idx int32 [T,k] in descending score,
    gate_w float32 [T,k], logits float64 [T,E]).

    The value in (0,1) of each expert is softmax(l) over all E experts.  The k highest are
    taken on the logits (softmax is monotone), ties going to the lower index.  renorm=1 divides
    the k gate values by their sum; renorm=0 keeps the raw softmax values."""
    l = router_logits(x, W_g, b)
    T, E = l.shape
    if not (1 <= k <= E):
        raise ValueError("k out of range")
    order = np.argsort(-l, axis=1, kind="stable")      # stable: equal logits keep index order
    idx = order[:, :k]
    p = np.exp(l - l.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, idx, axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return idx.astype(np.int32), w.astype(np.float32), l


def decision_gaps(logits: np.ndarray, k: int) -> np.ndarray:
    """Per token, the smallest gap between consecutive sorted logits at ranks 1..k+1 (the k
    comparisons that decide the top-k set and its order)."""
    s = -np.sort(-logits, axis=1)
    kk = min(k + 1, s.shape[1])
    return (s[:, : kk - 1] - s[:, 1:kk]).min(axis=1)


# ----------------------------------------------------------------------------- step 4: grouping
def permute(expert_idx: np.ndarray, E: int) -> Dict[str, np.ndarray]:
    """Group the A = T*k assignments by expert, keeping ascending assignment order inside each
    expert (a stable counting sort written out from its definition):

      counts[e]   = #{a : idx[a] = e}
      offsets[0]  = 0, offsets[e+1] = offsets[e] + counts[e]
      pos(a)      = offsets[idx[a]] + #{a' < a : idx[a'] = idx[a]}
      perm[pos(a)] = a,  inv_perm[a] = pos(a)
    """
    flat = np.asarray(expert_idx, dtype=np.int64).reshape(-1)
    A = flat.shape[0]
    if A and (flat.min() < 0 or flat.max() >= E):
        raise ValueError("expert id out of range")
    counts = np.zeros(E, dtype=np.int64)
    for a in range(A):
        counts[flat[a]] += 1
    offsets = np.zeros(E + 1, dtype=np.int64)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    seen = np.zeros(E, dtype=np.int64)
    perm = np.empty(A, dtype=np.int64)
    inv_perm = np.empty(A, dtype=np.int64)
    for a in range(A):
        e = flat[a]
        pos = offsets[e] + seen[e]
        seen[e] += 1
        perm[pos] = a
        inv_perm[a] = pos
    return {"counts": counts.astype(np.int32), "offsets": offsets.astype(np.int32),
            "perm": perm.astype(np.int32), "inv_perm": inv_perm.astype(np.int32)}


def gather_rows(x: np.ndarray, perm: np.ndarray, k: int) -> np.ndarray:
    """x_perm[r,:] = x[perm[r] div k, :] -- a bit copy, any dtype."""
    return np.asarray(x)[np.asarray(perm, dtype=np.int64) // k]


# ----------------------------------------------------------------------------- step 5: experts
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn(x_rows: np.ndarray, weights: Dict[str, np.ndarray], act: str,
               h_round: Optional[str] = None) -> np.ndarray:
    """One expert on a block of rows, float64 (section 4.4: x W1 W2, activation between).
    act="relu":   y = max(0, x W1) W2           weights: W1 [d,F], W2 [F,d]
    act="swiglu": y = (silu(x Wg) * (x Wu)) Wd  weights: Wg, Wu [d,F], Wd [F,d]
    h_round="bf16" / "f16" rounds the hidden activations to bfloat16 / IEEE half (saturating at
    +-65504) before the second product; that is a diagnostic that mimics a 16-bit intermediate,
    not the definition."""
    x = to_f64(x_rows)
    if act == "relu":
        h = np.maximum(x @ to_f64(weights["W1"]), 0.0)
        w_out = weights["W2"]
    elif act == "swiglu":
        h = silu(x @ to_f64(weights["Wg"])) * (x @ to_f64(weights["Wu"]))
        w_out = weights["Wd"]
    else:
        raise ValueError(act)
    if h_round == "bf16":
        h = round_to_bf16(h)
    elif h_round == "f16":
        # half with saturation: values beyond the largest half (65504) are kept at +-65504
        h = np.clip(h, -65504.0, 65504.0).astype(np.float16).astype(np.float64)   # float64 -> half directly, ties to even
    elif h_round is not None:
        raise ValueError(h_round)
    return h @ to_f64(w_out)


def _expert_slice(weights: Dict[str, np.ndarray], e: int) -> Dict[str, np.ndarray]:
    return {n: a[e] for n, a in weights.items()}


def moe_layer(x: np.ndarray, expert_idx: np.ndarray, gate_w: np.ndarray,
              weights: Dict[str, np.ndarray], act: str,
              shared: Optional[Dict[str, np.ndarray]] = None,
              tokens: Optional[Sequence[int]] = None, h_round: Optional[str] = None) -> np.ndarray:
    """y[t] = sum_{j<k} gate_w[t,j] * FFN_{idx[t,j]}(x[t])  (+ FFN_shared(x[t])),  float64.

    `weights` holds stacked per-expert matrices ([E, ...]).  `tokens` restricts the computation
    to a subset of token ids (rows of the result follow that order); the definition is per
    token, so a subset needs nothing else."""
    idx = np.asarray(expert_idx)
    T, k = idx.shape
    tok = np.arange(T) if tokens is None else np.asarray(tokens, dtype=np.int64)
    xs = np.asarray(x)[tok]
    idx_s = idx[tok]
    w_s = np.asarray(gate_w, dtype=np.float64)[tok]
    d = xs.shape[1]
    y = np.zeros((tok.shape[0], d), dtype=np.float64)
    E = next(iter(weights.values())).shape[0]
    for j in range(k):                      # fixed j order, as in the sum above
        for e in range(E):
            rows = np.nonzero(idx_s[:, j] == e)[0]
            if rows.size == 0:
                continue
            y[rows] += w_s[rows, j, None] * expert_ffn(xs[rows], _expert_slice(weights, e), act, h_round)
    if shared is not None:
        y += expert_ffn(xs, shared, "swiglu", h_round)
    return y


def grouped_ffn(x_perm: np.ndarray, offsets: np.ndarray, weights: Dict[str, np.ndarray],
                act: str, h_round: Optional[str] = None) -> np.ndarray:
    """Expert FFN on rows already grouped by expert: rows [offsets[e], offsets[e+1]) go through
    expert e.  Used to check the grouped-FFN stage on its own."""
    off = np.asarray(offsets, dtype=np.int64)
    d_out = (weights["W2"] if act == "relu" else weights["Wd"]).shape[2]
    y = np.zeros((x_perm.shape[0], d_out), dtype=np.float64)
    for e in range(off.shape[0] - 1):
        if off[e + 1] > off[e]:
            y[off[e]:off[e + 1]] = expert_ffn(x_perm[off[e]:off[e + 1]], _expert_slice(weights, e), act, h_round)
    return y


# ----------------------------------------------------------------------------- step 6: combine
def combine(y_perm: np.ndarray, inv_perm: np.ndarray, gate_w: np.ndarray,
            shared: Optional[np.ndarray] = None) -> np.ndarray:
    """y[t] = sum_{j<k} gate_w[t,j] * y_perm[inv_perm[t*k+j]] (+ shared[t]), float64."""
    gw = np.asarray(gate_w, dtype=np.float64)
    T, k = gw.shape
    yp = to_f64(y_perm)
    ip = np.asarray(inv_perm, dtype=np.int64).reshape(T, k)
    y = np.zeros((T, yp.shape[1]), dtype=np.float64)
    for j in range(k):
        y += gw[:, j, None] * yp[ip[:, j]]
    if shared is not None:
        y += to_f64(shared)
    return y


# ----------------------------------------------------------------------------- Alg. 2
def initial_assign(m_all: np.ndarray, home: Sequence[int], G: int) -> np.ndarray:
    """S_initial[g_from, e, g_to] (Alg. 1 step 3): every token of expert e coming from GPU
    g_from goes to the GPU that houses e.  m_all[g_from, e] = token counts, home[e] = GPU."""
    m_all = np.asarray(m_all, dtype=np.int64)
    G_src, E = m_all.shape
    S = np.zeros((G_src, E, G), dtype=np.int64)
    for g in range(G_src):
        for e in range(E):
            S[g, e, home[e]] = m_all[g, e]
    return S


class _NoMove(Exception):
    """Why the greedy loop of Alg. 2 ends: `reason` is one of "balanced" (no destination above the
    floor average), "small" (the chosen block holds fewer than q tokens) and "no_room" (the
    emptiest destination is the donor itself, or cannot take q tokens and stay at the average)."""

    def __init__(self, reason: str):
        super().__init__(reason)
        self.reason = reason


def _first_largest(values) -> int:
    """Index of the largest value, the lowest index among equals."""
    best = 0
    for i, v in enumerate(values):
        if v > values[best]:
            best = i
    return best


def _first_smallest(values) -> int:
    best = 0
    for i, v in enumerate(values):
        if v < values[best]:
            best = i
    return best


def pick_move(S: np.ndarray, load, average: int, q: int):
    """One decision of Alg. 2 on the state (S, load), with load[g] = tokens bound for GPU g.
    Returns (source, expert, donor, receiver, tokens) or raises _NoMove.

    The donor is the fullest destination.  Of the sources feeding it, the one whose tokens for
    the donor, summed over ALL experts, are the most is taken; of that source's experts, the one
    with the most tokens for the donor.  That single (source, expert) block is the candidate: it
    must hold q tokens.  The receiver is the emptiest destination and must be able to take q
    tokens without passing the average; it takes the block, or as much of it as brings it to the
    average (section 4.2)."""
    G_src, E, G = S.shape
    if not any(t > average for t in load):
        raise _NoMove("balanced")
    donor = _first_largest(load)
    per_source = [sum(int(S[s, e, donor]) for e in range(E)) for s in range(G_src)]
    source = _first_largest(per_source)
    expert = _first_largest([int(S[source, e, donor]) for e in range(E)])
    block = int(S[source, expert, donor])
    if block < q:
        raise _NoMove("small")
    receiver = _first_smallest(load)
    room = average - load[receiver]
    if receiver == donor or room < q:
        raise _NoMove("no_room")
    return source, expert, donor, receiver, min(block, room)


def rebalance(S_initial: np.ndarray, q: int, max_iters: int = 1_000_000, moves: Optional[list] = None
              ) -> np.ndarray:
    """Token rebalancing, Alg. 2 / section 4.2.  S[g_from, e, g_to] int64; q >= 1 is the transfer
    threshold.  The average is the floor of total / |G|.  Every "most" / "least" takes the lowest
    index among equals.  `moves`, if given, receives every transfer as
    (source, expert, donor, receiver, tokens) in the order they are made."""
    if q < 1:
        raise ValueError("q must be >= 1 (with q = 0 the loop can move zero tokens forever)")
    S = np.array(S_initial, dtype=np.int64, copy=True)
    G = S.shape[2]
    load = [int(S[:, :, g].sum()) for g in range(G)]
    average = sum(load) // G
    for _ in range(max_iters):
        try:
            source, expert, donor, receiver, n = pick_move(S, load, average, q)
        except _NoMove:
            break
        S[source, expert, donor] -= n
        S[source, expert, receiver] += n
        load[donor] -= n
        load[receiver] += n
        if moves is not None:
            moves.append((source, expert, donor, receiver, n))
    return S


# ----------------------------------------------------------------------------- threshold q
def expert_bytes(m: int, p: int, d_type: int) -> int:
    """|E| = (mp + pm) d_type, Eq. 2."""
    return (m * p + p * m) * d_type


def expert_flops(q: int, m: int, p: int) -> int:
    """|O| = q p (2m-1) + q m (2p-1), Eq. 3."""
    return q * p * (2 * m - 1) + q * m * (2 * p - 1)


def token_threshold_q(phi: float, d_type: int, beta: float) -> float:
    """Eq. 4: q > phi d_type / (2 beta)."""
    return phi * d_type / (2.0 * beta)


def token_threshold_q_exact(phi: float, d_type: int, beta: float, m: int, p: int) -> float:
    """The bound before the small terms are dropped (appendix B, third line): the q at which
    |O|/phi = |E|/beta."""
    return (expert_bytes(m, p, d_type) / beta) * phi / (p * (2 * m - 1) + m * (2 * p - 1))


# ----------------------------------------------------------------------------- one-GPU schedule
# The library runs Alg. 2 with the GPU's XCDs ("bins") in the role of the paper's GPUs and one
# source (G_src = 1), so S is [E, n_bins].  Two of its policies are the paper's own
# (schedule_harmoeny, schedule_static, schedule_even_split); schedule_balanced is this build's
# variant of Alg. 2 in units of tiles and is DEFINED by the function below (no paper counterpart
# to pin it to beyond a hand-worked case, the invariants in the tests, and its by_cost=False
# form, which is Alg. 2).

def contiguous_home(E: int, G: int):
    """Experts in contiguous blocks per GPU (Fig. 2 of the paper: experts 1,2 on GPU 0, ...)."""
    return [(e * G) // E for e in range(E)]


def round_robin_home(E: int, G: int):
    """Experts dealt to the GPUs in turn (section 5.3.2, policy 1): expert e lives on GPU e mod G."""
    return [e % G for e in range(E)]


def schedule_static(counts, G: int) -> np.ndarray:
    counts = np.asarray(counts, dtype=np.int64)
    return initial_assign(counts[None, :], contiguous_home(len(counts), G), G)[0]


def schedule_round_robin(counts, G: int) -> np.ndarray:
    """Round-robin policy (section 5.3.2, policy 1): experts dealt to the GPUs in turn, every
    token goes to the GPU that houses its expert, whatever the imbalance."""
    counts = np.asarray(counts, dtype=np.int64)
    return initial_assign(counts[None, :], round_robin_home(len(counts), G), G)[0]


def schedule_harmoeny(counts, G: int, q: int) -> np.ndarray:
    """Alg. 2 as printed, one source GPU, experts starting in contiguous blocks."""
    counts = np.asarray(counts, dtype=np.int64)
    S0 = initial_assign(counts[None, :], contiguous_home(len(counts), G), G)
    return rebalance(S0, q)[0]


def schedule_even_split(counts, G: int) -> np.ndarray:
    """Even Split (section 5.3.2): a tokens of an expert over G GPUs -> a/G each; the remainder
    of the integer division goes one token each to the lowest-numbered GPUs (the paper's a/4
    example leaves the remainder open)."""
    counts = np.asarray(counts, dtype=np.int64)
    S = np.zeros((len(counts), G), dtype=np.int64)
    for e, a in enumerate(counts):
        for g in range(G):
            S[e, g] = a // G + (1 if g < a % G else 0)
    return S


def schedule_balanced(counts, G: int, q: int, tile_m: int, by_cost: bool = True) -> np.ndarray:
    """This build's default schedule (by_cost=True): the bins get equal numbers of TILES.
    A block of n rows of one expert on one bin weighs ceil(n / tile_m): the kernels work tile by
    tile, and a tile costs about the same whether its rows are many (arithmetic) or few (the
    fetch of the expert's weights, section 4.4).
    1. initialAssign: experts in order of falling weight (equal weights: rising id), each whole
       onto the bin with the least weight so far (lowest bin among equals).
    2. Alg. 2's loop in tiles: take the most and the least loaded bin (lowest index among
       equals); stop when they differ by at most one tile; otherwise move m = min(tiles of the
       block, floor(difference / 2)) tiles of the largest block (most rows, lowest expert among
       equals) of the most loaded bin to the least loaded one: the whole block if m covers it,
       else m * tile_m rows.  q is not used.
    by_cost=False: weights are row counts and step 2 is rebalance() itself (one source)."""
    counts = np.asarray(counts, dtype=np.int64)
    E = len(counts)
    tiles_of = lambda n: (int(n) + tile_m - 1) // tile_m
    w = tiles_of if by_cost else (lambda n: int(n))
    S = np.zeros((E, G), dtype=np.int64)
    order = sorted(range(E), key=lambda e: (-w(counts[e]), e))
    t_g = np.zeros(G, dtype=np.int64)
    for e in order:
        if w(counts[e]) == 0:
            break
        g = int(np.argmin(t_g))
        S[e, g] = counts[e]
        t_g[g] += w(counts[e])
    if by_cost:
        for _ in range(E * G + 16):
            g_max, g_min = int(np.argmax(t_g)), int(np.argmin(t_g))
            diff = int(t_g[g_max] - t_g[g_min])
            if diff <= 1:
                break
            e_max = int(np.argmax(S[:, g_max]))
            n_from, n_to = int(S[e_max, g_max]), int(S[e_max, g_min])
            m = min(tiles_of(n_from), diff // 2)
            t_s = n_from if m == tiles_of(n_from) else m * tile_m
            t_g[g_max] -= tiles_of(n_from) - tiles_of(n_from - t_s)
            t_g[g_min] += tiles_of(n_to + t_s) - tiles_of(n_to)
            S[e_max, g_max] = n_from - t_s
            S[e_max, g_min] = n_to + t_s
        return S
    return rebalance(S[None, :, :], q)[0]


def block_order(rows_of: dict, tile_m: int):
    """The order in which one bin lists its blocks (rows_of: expert -> rows of that expert on
    the bin, all positive).  The paper does not order the work inside a GPU (Alg. 1 step 5 just
    runs the experts); this is the library's launch order.  Blocks of more than one tile
    ("long") and the others ("short") are each ordered by falling row count, then expert id.
    If the long ones outnumber the short ones, or one kind is missing, the long ones come first.
    Otherwise the two lists are merged evenly: the i-th of L long blocks has the key (2i+1)/L,
    the j-th of M short ones (2j+1)/M; rising key, a long block first among equal keys."""
    by_size = sorted(rows_of, key=lambda e: (-rows_of[e], e))
    long_ = [e for e in by_size if rows_of[e] > tile_m]
    short = [e for e in by_size if rows_of[e] <= tile_m]
    if not long_ or not short or len(long_) > len(short):
        return long_ + short
    keyed = [(Fraction(2 * i + 1, len(long_)), 0, e) for i, e in enumerate(long_)]
    keyed += [(Fraction(2 * j + 1, len(short)), 1, e) for j, e in enumerate(short)]
    return [e for _, _, e in sorted(keyed)]


def tiles_from_schedule(S: np.ndarray, offsets, tile_m: int):
    """The tile table a schedule S [E, n_bins] stands for: bin after bin; inside a bin the
    blocks in block_order(); a block's rows are the expert's rows after those of
    lower-numbered bins, cut into tiles of at most tile_m rows.
    Returns (tiles [n,4] int32 = expert,row_begin,row_count,bin ; bin_start [G+1])."""
    S = np.asarray(S, dtype=np.int64)
    E, G = S.shape
    before = np.concatenate([np.zeros((E, 1), dtype=np.int64), np.cumsum(S, axis=1)[:, :-1]], axis=1)
    tiles, bin_start = [], [0]
    for g in range(G):
        for e in block_order({e: int(S[e, g]) for e in range(E) if S[e, g] > 0}, tile_m):
            row, left = int(offsets[e] + before[e, g]), int(S[e, g])
            while left > 0:
                rc = min(tile_m, left)
                tiles.append((e, row, rc, g))
                row += rc
                left -= rc
        bin_start.append(len(tiles))
    return np.array(tiles, dtype=np.int32).reshape(-1, 4), np.array(bin_start, dtype=np.int32)


def validate_tiles(tiles: np.ndarray, bin_start: np.ndarray, counts, offsets, tile_m: int, G: int) -> None:
    """Raises AssertionError unless the table is a valid plan: bins contiguous and in order,
    every row of [0,A) in exactly one tile, no tile across an expert boundary or above tile_m."""
    counts = np.asarray(counts, dtype=np.int64)
    offsets = np.asarray(offsets, dtype=np.int64)
    A = int(offsets[-1])
    assert len(bin_start) == G + 1 and bin_start[0] == 0 and bin_start[-1] == len(tiles)
    assert np.all(np.diff(bin_start) >= 0)
    covered = np.zeros(A, dtype=np.int64)
    for g in range(G):
        for e, rb, rc, b in tiles[bin_start[g]:bin_start[g + 1]]:
            assert b == g and 0 < rc <= tile_m
            assert offsets[e] <= rb and rb + rc <= offsets[e + 1]
            covered[rb:rb + rc] += 1
    assert np.all(covered == 1)
