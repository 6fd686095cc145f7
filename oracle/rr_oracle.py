"""Plain fp64 CPU statement of the RRAttention prefill path.  TEST INFRASTRUCTURE ONLY.

This module exists to check the HIP library.  Only the tests, the smoke check
and the benchmark's CPU-baseline leg may import it; the product path never does.
It shares no code, table or helper with the HIP path.

Every function follows one passage of the paper (arxiv 2602.05853) and is kept
slow and literal on purpose: numpy fp64, one head at a time, no tiling, no
fusion.  Indices are 0-based everywhere.

Readings taken where the paper is silent or inconsistent (each one is repeated
at the function that applies it):
  R1  the stride-level softmax (Sec. 3.2, softmax equation) is causal: only key
      strides j <= i enter row i.  The equation as printed sums over all j, but
      the problem statement forbids blocks above the diagonal.
  R2  the key aggregate of a stride is the sum over the whole stride, also for
      the diagonal stride, whatever the sampled offset of the head is.
  R3  Top-tau compares the cumulative mass with tau times the row total (a row
      of block masses sums to B/S, not to 1).
  R4  the selected set is the minimal prefix, in descending mass order, whose
      cumulative mass is >= tau (the sentence before the selection equation);
      equal masses are ordered by smaller block index first.
  R5  the head index h of the sampling rule is the 0-based query-head index;
      with grouped-query attention query head h reads KV head h // (Hq/Hkv).
  R6  masked logits are excluded from the softmax (the "odot M" of the
      block-sparse attention equation means "keep only where M = 1").
  R7  S | B is required.  L is free: as in the problem statement (Sec. 2.1) there
      are ceil(L/B) blocks, the last one possibly partial, and floor(L/S) strides
      (Sec. 3.1); positions after the last complete stride belong to no stride
      (they are never sampled and never scored) but are attended like any other.
      A query block without a single complete stride has no estimate: it keeps
      every causal block.
  R8  ablation variants (Sec. 4, round-robin strategy table and last-query-block
      table) are named but not defined by formulas.  Taken here: the sampled
      offset is S - 1 - (phase mod S) with phase = h (head round-robin, the
      method), 0 (no round-robin), l (layer round-robin, l = layer index) or
      h + l (hybrid); "sink & recent block" protection adds the first
      `sink_blocks` key blocks and the `recent_blocks` key blocks ending at the
      diagonal to every row after Top-tau (a union, like the last-query-block
      protection of Sec. 3.3).

  R9  block selection accuracy (appendix): the ground-truth key set is taken
      greedily by descending attention, equal values by smaller position first
      (one of the smallest sets); the predicted set of query i is clipped to
      positions j <= i; a query with an empty predicted set has precision 0.
  R11 alternative to R2, selectable (diagonal = "token"): in the sampled query's own
      stride only the keys up to the query's position are summed.
  R12 decode-stage extension (the paper's "Future Work" names it without an algorithm; its experiments
      decode densely).  Taken here: a step brings the last Lq >= 1 positions of an L-token context as
      queries, at ANY offset q0 = L - Lq (one token, a few speculative tokens, a chunk that starts inside
      a block); keys are the whole context.  The method is applied as stated to what exists: the query
      blocks touched by the step are floor(q0/B) .. ceil(L/B)-1, a row's estimate uses those of its
      sampled positions (Sec. 3.1) that lie inside the step (p >= q0) and in a complete stride (R7), and
      a row left without any sampled query keeps every causal block (R7's rule) -- so a one-token step
      is dense, as in the paper's experiments, unless the token is its head's sampled position of a stride
      that it completes.  Attention rows are those of Sec. 2.1 for the positions q0 .. L-1.  A step that
      starts at a block boundary is chunked prefill; q0 = 0 is the method itself.  Parity against the
      paper: unpinned (no definition there); pinned against these reductions and hand-written loops.
  R10 packed sequences: the method is stated for one sequence (Sec. 2.1, 3.1-3.3),
      so a batch of sequences laid back to back is treated sequence by sequence;
      each holds a whole number of blocks.  The packed mask is block diagonal.

Parity status: every function below is pinned by tests/test_oracle_pins.py
(library softmax attention, S = 1 reduction, constant-key closed form,
stride-constant keys, NaN-poisoned unsampled rows, subset brute force, hand-worked
offset tables, union identity of the protections, closed forms of precision /
recall on uniform and one-hot attention).  The offset formulas of the ablation
variants (R8) are this build's reading, not the paper's text: parity unpinned
against the paper for those.  The numeric masks of the five benchmark workloads
have no external pin: there the oracle is the definition.
"""
from __future__ import annotations

import math
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------
# Sec. 3.1  query sampling with the head round-robin rule
# ----------------------------------------------------------------------------

OFFSET_MODES = ("head", "fixed", "layer", "hybrid")


def offset_phase(h: int, mode: str = "head", layer: int = 0) -> int:
    """The quantity reduced mod S in the sampling rule.  "head" is Sec. 3.1; the others are reading R8."""
    if mode == "head":
        return h
    if mode == "fixed":
        return 0
    if mode == "layer":
        return layer
    if mode == "hybrid":
        return h + layer
    raise ValueError(f"unknown offset mode {mode!r}")


def sample_positions(L: int, S: int, h: int, mode: str = "head", layer: int = 0) -> np.ndarray:
    """Sec. 3.1, sampling equation: P(i, h) = i*S + (S - 1 - (h mod S)), i in [0, floor(L/S)).

    With a mode other than "head", h is replaced by offset_phase(h, mode, layer) (reading R8)."""
    i = np.arange(L // S)
    return i * S + (S - 1 - (offset_phase(h, mode, layer) % S))


# ----------------------------------------------------------------------------
# Sec. 3.2  stride-level importance
# ----------------------------------------------------------------------------

def stride_key_sums(Kg: np.ndarray, S: int) -> np.ndarray:
    """Inner sum of the importance equation (Sec. 3.2): sum of the keys of stride j.  Reading R2."""
    L, d = Kg.shape
    Ls = L // S
    # row j of the result = sum of rows j*S .. (j+1)*S - 1
    return Kg[: Ls * S].astype(np.float64).reshape(Ls, S, d).sum(axis=1)


def stride_scores(Qh: np.ndarray, Kg: np.ndarray, S: int, h: int, mode: str = "head", layer: int = 0,
                  diagonal: str = "stride") -> np.ndarray:
    """Importance equation (Sec. 3.2): I[i, j] = Q[P(i,h)] . (sum of stride j keys) / (S sqrt(d)).

    diagonal = "stride" is reading R2.  diagonal = "token" is the alternative reading (R11): in the
    query's own stride (j = i) only the keys at positions <= P(i, h) are summed, so that no sampled query
    is scored against a key that follows it; the factor 1 / (S sqrt(d)) stays as printed."""
    L, d = Qh.shape
    pos = sample_positions(L, S, h, mode, layer)
    qs = Qh[pos].astype(np.float64)
    ksum = stride_key_sums(Kg, S)
    I = (qs @ ksum.T) / (S * math.sqrt(d))
    if diagonal == "token":
        for i in range(L // S):
            visible = Kg[i * S: pos[i] + 1].astype(np.float64).sum(axis=0)
            I[i, i] = (qs[i] @ visible) / (S * math.sqrt(d))
    elif diagonal != "stride":
        raise ValueError(f"unknown diagonal rule {diagonal!r}")
    return I


def stride_softmax(I: np.ndarray) -> np.ndarray:
    """Row softmax at stride granularity (Sec. 3.2), restricted to j <= i.  Reading R1."""
    Ls = I.shape[0]
    P = np.zeros_like(I)
    for i in range(Ls):
        row = I[i, : i + 1]
        e = np.exp(row - row.max())
        P[i, : i + 1] = e / e.sum()
    return P


# ----------------------------------------------------------------------------
# Sec. 3.3  block mass and Top-tau selection
# ----------------------------------------------------------------------------

def block_mass(P: np.ndarray, R: int, Nb: Optional[int] = None) -> np.ndarray:
    """Block importance (Sec. 3.3): S[m, n] = sum of P over query strides of block m, key strides of block n.

    Nb > Ls / R (a partial last block, reading R7): the strides that do not exist contribute nothing."""
    Ls = P.shape[0]
    if Nb is None:
        Nb = Ls // R
    full = np.zeros((Nb * R, Nb * R), dtype=np.float64)
    full[:Ls, :Ls] = P
    # axis 0 -> (m, query stride inside block m), axis 1 -> (n, key stride inside block n)
    return full.reshape(Nb, R, Nb, R).sum(axis=(1, 3))


def top_tau_row(mass: np.ndarray, tau: float) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Top-tau selection for one query block (Sec. 3.3).  Readings R3, R4.

    mass: block masses of the causal candidates n = 0..m of this row.
    Returns (selected flags, order, cumulative): `order` lists the candidates by
    descending mass (smaller index first among equals) and `cumulative[k]` is
    the normalised mass of order[0..k].
    """
    total = mass.sum()
    frac = mass / total
    order = np.argsort(-frac, kind="stable")
    cumulative = np.cumsum(frac[order])
    sel = np.zeros(mass.shape[0], dtype=bool)
    if tau >= 1.0:
        sel[:] = True
        return sel, order, cumulative
    reached = np.nonzero(cumulative >= tau)[0]
    k = int(reached[0]) + 1 if reached.size else mass.shape[0]
    sel[order[:k]] = True
    return sel, order, cumulative


def select_blocks(mass: np.ndarray, tau: float, protect_last: bool = True, sink_blocks: int = 0,
                  recent_blocks: int = 0):
    """Dynamic mask, then OR with the protected last query-block row (Sec. 3.3, last two equations).

    sink_blocks / recent_blocks (reading R8): key blocks n < sink_blocks and m - recent_blocks < n <= m
    are added to every row m after Top-tau.

    mass: [Nb, Nb] block masses of one head (zeros above the diagonal).
    Returns (mask uint8 [Nb, Nb], frac [Nb, Nb] normalised mass, margin [Nb, Nb]).
    margin[m, n] is |c - tau| where c is the normalised cumulative mass of the
    blocks ranked before n in row m: n is selected exactly when c < tau, so the
    margin says how far the decision for that block is from flipping.
    """
    Nb = mass.shape[0]
    mask = np.zeros((Nb, Nb), dtype=np.uint8)
    frac = np.zeros((Nb, Nb), dtype=np.float64)
    margin = np.full((Nb, Nb), np.inf, dtype=np.float64)
    for m in range(Nb):
        row = mass[m, : m + 1]
        if row.sum() == 0.0:               # no complete stride in this query block (reading R7): keep everything
            mask[m, : m + 1] = 1
            continue
        sel, order, cum = top_tau_row(row, tau)
        mask[m, : m + 1] = sel
        frac[m, : m + 1] = row / row.sum()
        before = np.concatenate(([0.0], cum[:-1]))
        margin[m, order] = np.abs(before - tau)
    if protect_last:
        mask[Nb - 1, :Nb] = 1
    for m in range(Nb):
        for n in range(m + 1):
            if n < sink_blocks or n > m - recent_blocks:
                mask[m, n] = 1
    return mask, frac, margin


def estimate_head(Qh: np.ndarray, Kg: np.ndarray, h: int, S: int, B: int, tau: float,
                  protect_last: bool = True, mode: str = "head", layer: int = 0,
                  sink_blocks: int = 0, recent_blocks: int = 0, diagonal: str = "stride"):
    """Pattern estimation for one query head: Sec. 3.1 -> 3.2 -> 3.3 in the paper's order."""
    L = Qh.shape[0]
    if B % S:
        raise ValueError("S | B is required (reading R7)")
    I = stride_scores(Qh, Kg, S, h, mode, layer, diagonal)
    P = stride_softmax(I)
    mass = block_mass(P, B // S, -(-L // B))
    return select_blocks(mass, tau, protect_last, sink_blocks, recent_blocks)


def estimate_row(Qh: np.ndarray, Kg: np.ndarray, h: int, m: int, S: int, B: int, tau: float,
                 protect_last: bool = True):
    """Row m of estimate_head's result alone (for lengths whose full stride matrix is too large to hold):
    the same passages applied to the R = B/S sampled queries of query block m only.

    Returns (mask row [m+1] uint8, frac row [m+1], margin row [m+1])."""
    L, d = Qh.shape
    R = B // S
    pos = sample_positions(L, S, h)[m * R:(m + 1) * R]            # Sec. 3.1
    ksum = stride_key_sums(Kg[: (m + 1) * B], S)                  # Sec. 3.2, strides 0 .. (m+1) R - 1
    I = (Qh[pos].astype(np.float64) @ ksum.T) / (S * math.sqrt(d))
    mass = np.zeros(m + 1, dtype=np.float64)
    for r in range(R):
        i = m * R + r
        row = I[r, : i + 1]                                       # causal at stride level (reading R1)
        e = np.exp(row - row.max())
        p = np.zeros((m + 1) * R, dtype=np.float64)
        p[: i + 1] = e / e.sum()
        mass += p.reshape(m + 1, R).sum(axis=1)                   # Sec. 3.3, block mass
    sel, order, cum = top_tau_row(mass, tau)
    margin = np.empty(m + 1, dtype=np.float64)
    margin[order] = np.abs(np.concatenate(([0.0], cum[:-1])) - tau)
    mask = sel.astype(np.uint8)
    if protect_last and (m + 1) * B == L:
        mask[:] = 1
    return mask, mass / mass.sum(), margin


def estimate(Q: np.ndarray, K: np.ndarray, S: int, B: int, tau: float, protect_last: bool = True,
             mode: str = "head", layer: int = 0, sink_blocks: int = 0, recent_blocks: int = 0,
             diagonal: str = "stride"):
    """rr_estimate for all heads.  Q [Hq, L, d], K [Hkv, L, d].  Reading R5 for the head mapping.

    Returns (mask [Hq, Nb, Nb] uint8, frac [Hq, Nb, Nb], margin [Hq, Nb, Nb]).
    """
    Hq, Hkv = Q.shape[0], K.shape[0]
    G = Hq // Hkv
    outs = [estimate_head(Q[h], K[h // G], h, S, B, tau, protect_last, mode, layer, sink_blocks, recent_blocks,
                          diagonal)
            for h in range(Hq)]
    return (np.stack([o[0] for o in outs]), np.stack([o[1] for o in outs]),
            np.stack([o[2] for o in outs]))


def estimate_step_head(Qh: np.ndarray, Kg: np.ndarray, h: int, q0: int, S: int, B: int, tau: float,
                       protect_last: bool = True, mode: str = "head", layer: int = 0,
                       sink_blocks: int = 0, recent_blocks: int = 0, diagonal: str = "stride"):
    """Pattern estimation of one head for a step whose queries are the positions q0 .. L-1 (reading R12).

    Qh is indexed by absolute position; rows before q0 are not part of the step and are never read.
    Returns the rows floor(q0/B) .. Nb-1 of (mask, frac, margin), each [rows, Nb]."""
    L = Qh.shape[0]
    if B % S:
        raise ValueError("S | B is required (reading R7)")
    Qstep = np.zeros_like(Qh, dtype=np.float64)
    Qstep[q0:] = Qh[q0:]                                          # nothing before the step is looked at
    I = stride_scores(Qstep, Kg, S, h, mode, layer, diagonal)     # Sec. 3.2
    P = stride_softmax(I)
    usable = sample_positions(L, S, h, mode, layer) >= q0         # Sec. 3.1 positions that the step holds
    P[~usable] = 0.0                                              # the others do not exist for this step
    mass = block_mass(P, B // S, -(-L // B))                      # Sec. 3.3
    mask, frac, margin = select_blocks(mass, tau, protect_last, sink_blocks, recent_blocks)
    first = q0 // B
    return mask[first:], frac[first:], margin[first:]


def estimate_step(Q: np.ndarray, K: np.ndarray, q0: int, S: int, B: int, tau: float, protect_last: bool = True,
                  **kw):
    """estimate_step_head for all heads: (mask, frac, margin), each [Hq, rows, Nb], rows = Nb - floor(q0/B)."""
    Hq, Hkv = Q.shape[0], K.shape[0]
    G = Hq // Hkv
    outs = [estimate_step_head(Q[h], K[h // G], h, q0, S, B, tau, protect_last, **kw) for h in range(Hq)]
    return (np.stack([o[0] for o in outs]), np.stack([o[1] for o in outs]), np.stack([o[2] for o in outs]))


def sequence_block_ranges(blocks_per_sequence: Sequence[int]) -> List[Tuple[int, int]]:
    """[first block, one past the last block) of every sequence of a packed batch (reading R10)."""
    ranges, at = [], 0
    for nb in blocks_per_sequence:
        ranges.append((at, at + int(nb)))
        at += int(nb)
    return ranges


def estimate_packed(Q: np.ndarray, K: np.ndarray, S: int, B: int, tau: float,
                    blocks_per_sequence: Sequence[int], protect_last: bool = True, mode: str = "head",
                    layer: int = 0, sink_blocks: int = 0, recent_blocks: int = 0, diagonal: str = "stride"):
    """Pattern estimation of sequences packed back to back along the position axis (reading R10).

    Every sequence is cut out and estimated exactly as `estimate` does for a single prompt (positions,
    strides and blocks counted from the sequence's own start; its own last query block protected); its
    [Nb_s, Nb_s] results are placed on the diagonal of the packed [Hq, Nb, Nb] arrays.  Nothing is
    selected across sequences; margin is +inf there.
    """
    Hq, L = Q.shape[0], Q.shape[1]
    Nb = -(-L // B)                        # the last sequence may end inside its last block (reading R7)
    if sum(int(n) for n in blocks_per_sequence) != Nb:
        raise ValueError("the sequences must fill the packed length")
    mask = np.zeros((Hq, Nb, Nb), dtype=np.uint8)
    frac = np.zeros((Hq, Nb, Nb), dtype=np.float64)
    margin = np.full((Hq, Nb, Nb), np.inf, dtype=np.float64)
    for (b0, b1) in sequence_block_ranges(blocks_per_sequence):
        sl = slice(b0 * B, min(b1 * B, L))
        mk, fr, mg = estimate(Q[:, sl], K[:, sl], S, B, tau, protect_last, mode, layer, sink_blocks, recent_blocks,
                              diagonal)
        mask[:, b0:b1, b0:b1] = mk
        frac[:, b0:b1, b0:b1] = fr
        margin[:, b0:b1, b0:b1] = mg
    return mask, frac, margin


def packed_causal_block_mask(Hq: int, blocks_per_sequence: Sequence[int]) -> np.ndarray:
    """Dense baseline of a packed batch: every causal block of a row's own sequence."""
    Nb = sum(int(n) for n in blocks_per_sequence)
    mask = np.zeros((Hq, Nb, Nb), dtype=np.uint8)
    for (b0, b1) in sequence_block_ranges(blocks_per_sequence):
        mask[:, b0:b1, b0:b1] = np.tril(np.ones((b1 - b0, b1 - b0), dtype=np.uint8))
    return mask


# ----------------------------------------------------------------------------
# Sec. 2.1  block-sparse causal attention
# ----------------------------------------------------------------------------

def attention_row_block(Qh: np.ndarray, Kg: np.ndarray, Vg: np.ndarray, mask_row: np.ndarray,
                        m: int, B: int) -> Tuple[np.ndarray, np.ndarray]:
    """Block-sparse attention (Sec. 2.1, first two equations) for the queries of block m.

    Token (i, j) takes part iff mask_row[floor(j/B)] = 1 and j <= i (reading R6:
    all other logits are left out of the softmax).  Returns (O [B, d], lse [B]);
    a query with no admissible key gets O = 0 and lse = -inf.
    """
    L, d = Qh.shape
    q = Qh[m * B:(m + 1) * B].astype(np.float64)           # fewer than B rows in a partial last block
    rows = q.shape[0]
    # key positions of the selected causal blocks; every other position has M = 0
    blocks = [n for n in range(m + 1) if mask_row[n]]
    j_idx = np.concatenate([np.arange(n * B, min((n + 1) * B, L)) for n in blocks]) if blocks \
        else np.zeros(0, dtype=np.int64)
    k = Kg[j_idx].astype(np.float64)
    v = Vg[j_idx].astype(np.float64)
    logits = (q @ k.T) / math.sqrt(d)
    i_idx = m * B + np.arange(rows)[:, None]
    allowed = j_idx[None, :] <= i_idx
    logits = np.where(allowed, logits, -np.inf)
    out = np.zeros((rows, d), dtype=np.float64)
    lse = np.full(rows, -np.inf, dtype=np.float64)
    for r in range(rows):
        if not allowed[r].any():
            continue
        mx = logits[r].max()
        e = np.exp(logits[r] - mx)
        s = e.sum()
        out[r] = (e / s) @ v
        lse[r] = mx + math.log(s)
    return out, lse


def sparse_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, mask: np.ndarray, B: int,
                     rows: Optional[Iterable[Tuple[int, int]]] = None):
    """rr_sparse_attn: O [Hq, L, d] and lse [Hq, L] for the given block mask [Hq, Nb, Nb].

    With `rows` (pairs (h, m)) only those query blocks are evaluated and the
    result is a dict {(h, m): (O block, lse block)}.
    """
    Hq, L, d = Q.shape
    G = Hq // K.shape[0]
    Nb = -(-L // B)
    if rows is not None:
        return {(h, m): attention_row_block(Q[h], K[h // G], V[h // G], mask[h, m], m, B)
                for (h, m) in rows}
    O = np.zeros((Hq, L, d), dtype=np.float64)
    lse = np.zeros((Hq, L), dtype=np.float64)
    for h in range(Hq):
        for m in range(Nb):
            o, l = attention_row_block(Q[h], K[h // G], V[h // G], mask[h, m], m, B)
            O[h, m * B:(m + 1) * B] = o
            lse[h, m * B:(m + 1) * B] = l
    return O, lse


def causal_block_mask(Hq: int, Nb: int) -> np.ndarray:
    """All causal blocks selected: the dense baseline expressed as a block mask."""
    return np.broadcast_to(np.tril(np.ones((Nb, Nb), dtype=np.uint8)), (Hq, Nb, Nb)).copy()


def dense_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, B: int,
                    rows: Optional[Iterable[Tuple[int, int]]] = None):
    """rr_dense_attn: full causal softmax attention = the sparse definition with every causal block kept."""
    Hq, L, _ = Q.shape
    return sparse_attention(Q, K, V, causal_block_mask(Hq, -(-L // B)), B, rows)


# ----------------------------------------------------------------------------
# Appendix "Block Selection Accuracy Analysis": precision / recall / F1 of a block mask
# ----------------------------------------------------------------------------

def attention_row(Qh: np.ndarray, Kg: np.ndarray, i: int) -> np.ndarray:
    """Row i of the full causal attention matrix A (appendix, problem formulation): softmax over j <= i."""
    d = Qh.shape[1]
    s = Kg[: i + 1].astype(np.float64) @ Qh[i].astype(np.float64) / math.sqrt(d)
    e = np.exp(s - s.max())
    return e / e.sum()


def important_key_set(a_row: np.ndarray, tau: float) -> np.ndarray:
    """Ground-truth key set of one query (appendix, first equation): a smallest set of positions whose
    attention sums to >= tau.  Taken greedily by descending attention, equal values by smaller position
    first, which is one of the arg-min sets (any smallest set has the same size).  Returns a boolean
    array over the row's positions."""
    order = np.argsort(-a_row, kind="stable")
    cum = np.cumsum(a_row[order])
    reached = np.nonzero(cum >= tau)[0]
    k = int(reached[0]) + 1 if reached.size else a_row.shape[0]
    keep = np.zeros(a_row.shape[0], dtype=bool)
    keep[order[:k]] = True
    return keep


def selection_accuracy_query(Qh: np.ndarray, Kg: np.ndarray, mask_row: np.ndarray, i: int, B: int, tau: float):
    """Precision and recall terms of query i (appendix, second to fourth equations): the predicted key
    set is every position j <= i of the selected blocks of the query's block row.
    Returns (|K n K*|, |K|, |K*|)."""
    star = important_key_set(attention_row(Qh, Kg, i), tau)
    j = np.arange(i + 1)
    pred = mask_row[j // B].astype(bool)
    return int((pred & star).sum()), int(pred.sum()), int(star.sum())


def selection_accuracy(Q: np.ndarray, K: np.ndarray, mask: np.ndarray, B: int, tau: float, step: int = 1):
    """Precision, recall and F1 per head (appendix, last three equations), averaged over the query
    positions i = step-1, 2*step-1, ... (step = 1: every position, as in the paper).
    Returns an array [Hq, 3]; a query with an empty predicted set contributes precision 0."""
    Hq, L, _ = Q.shape
    G = Hq // K.shape[0]
    out = np.zeros((Hq, 3))
    for h in range(Hq):
        ps, rs, n = 0.0, 0.0, 0
        for i in range(step - 1, L, step):
            inter, pred, star = selection_accuracy_query(Q[h], K[h // G], mask[h, i // B], i, B, tau)
            ps += inter / pred if pred else 0.0
            rs += inter / star
            n += 1
        p, r = ps / n, rs / n
        out[h] = (p, r, 2 * p * r / (p + r) if p + r > 0 else 0.0)
    return out


# ----------------------------------------------------------------------------
# comparison rule for block masks (not part of the method: the parity bar)
# ----------------------------------------------------------------------------

def compare_masks(mask_ref: np.ndarray, margin_ref: np.ndarray, frac_ref: np.ndarray,
                  mask_test: np.ndarray, margin_tol: float = 1e-4, tie_tol: float = 1e-6):
    """Classify the disagreements between an oracle mask and a mask under test.

    A disagreeing block is `excused` when the oracle's decision for it sits
    within margin_tol of flipping (cumulative mass before it within margin_tol
    of tau); this is the only excuse.  Everything else is `failed`.
    `near_tie_rows` is information only: the number of rows whose failed blocks
    are one block dropped and one block added with masses within tie_tol of each
    other (such a row still counts as failed).
    """
    diff = mask_ref != mask_test
    excused = diff & (margin_ref < margin_tol)
    hard = diff & ~excused
    near_tie_rows = 0
    for h, m in {(h, m) for h, m, _ in zip(*np.nonzero(hard))}:
        cols = np.nonzero(diff[h, m])[0]
        if cols.size == 2 and mask_ref[h, m, cols[0]] != mask_ref[h, m, cols[1]] and \
                abs(frac_ref[h, m, cols[0]] - frac_ref[h, m, cols[1]]) < tie_tol:
            near_tie_rows += 1
    return {"mismatch": int(diff.sum()), "excused": int(excused.sum()),
            "near_tie_rows": near_tie_rows, "failed": int(hard.sum())}
