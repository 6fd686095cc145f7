"""The oracle against what the paper and the mathematics fix, and a mutation check of those pins."""
import importlib.util
import math
import os

import numpy as np
import pytest

from oracle import rr_oracle
import oracle_pins as pins


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(rr_oracle)


def _fresh_copy():
    spec = importlib.util.spec_from_file_location("rr_oracle_mutant", rr_oracle.__file__)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _mut_offset_ascending(o):
    o.sample_positions = lambda L, S, h, *a: np.arange(L // S) * S + (h % S)


def _mut_offset_ignores_head(o):
    o.sample_positions = lambda L, S, h, *a: np.arange(L // S) * S + (S - 1)


def _mut_key_window_shifted(o):
    def f(Kg, S):
        L, d = Kg.shape
        Ls = L // S
        Kr = np.roll(Kg.astype(np.float64), -1, axis=0)
        return Kr[: Ls * S].reshape(Ls, S, d).sum(axis=1)
    o.stride_key_sums = f


def _mut_missing_one_over_S(o):
    orig = o.stride_scores
    o.stride_scores = lambda Qh, Kg, S, h, *a, **kw: orig(Qh, Kg, S, h, *a, **kw) * S


def _mut_missing_sqrt_d(o):
    orig = o.stride_scores
    o.stride_scores = lambda Qh, Kg, S, h, *a, **kw: orig(Qh, Kg, S, h, *a, **kw) * math.sqrt(Qh.shape[1])


def _mut_noncausal_softmax(o):
    def f(I):
        e = np.exp(I - I.max(axis=1, keepdims=True))
        return e / e.sum(axis=1, keepdims=True)
    o.stride_softmax = f


def _mut_block_mass_transposed(o):
    orig = o.block_mass
    o.block_mass = lambda P, R, Nb=None: orig(P, R, Nb).T.copy()


def _mut_strict_threshold(o):
    def f(mass, tau):
        frac = mass / mass.sum()
        order = np.argsort(-frac, kind="stable")
        cum = np.cumsum(frac[order])
        sel = np.zeros(mass.shape[0], dtype=bool)
        reached = np.nonzero(cum > tau)[0]
        k = int(reached[0]) + 1 if reached.size else mass.shape[0]
        sel[order[:k]] = True
        return sel, order, cum
    o.top_tau_row = f


def _mut_unnormalised_threshold(o):
    def f(mass, tau):
        order = np.argsort(-mass, kind="stable")
        cum = np.cumsum(mass[order])
        sel = np.zeros(mass.shape[0], dtype=bool)
        reached = np.nonzero(cum >= tau)[0]
        k = int(reached[0]) + 1 if reached.size else mass.shape[0]
        sel[order[:k]] = True
        return sel, order, cum / mass.sum()
    o.top_tau_row = f


def _mut_ties_larger_index_first(o):
    orig = o.top_tau_row

    def f(mass, tau):
        sel, order, cum = orig(mass[::-1], tau)
        n = mass.shape[0]
        return sel[::-1].copy(), (n - 1 - order), cum
    o.top_tau_row = f


def _mut_no_protection(o):
    orig = o.select_blocks
    o.select_blocks = lambda mass, tau, protect_last=True, *a: orig(mass, tau, False, *a)


def _mut_hybrid_ignores_layer(o):
    orig = o.offset_phase
    o.offset_phase = lambda h, mode="head", layer=0: h if mode == "hybrid" else orig(h, mode, layer)


def _mut_layer_mode_uses_head(o):
    orig = o.offset_phase
    o.offset_phase = lambda h, mode="head", layer=0: h + layer if mode == "layer" else orig(h, mode, layer)


def _mut_recent_excludes_diagonal(o):
    orig = o.select_blocks

    def f(mass, tau, protect_last=True, sink_blocks=0, recent_blocks=0):
        mask, frac, margin = orig(mass, tau, protect_last, sink_blocks, 0)
        Nb = mask.shape[0]
        for m in range(Nb):
            for n in range(m):
                if n >= m - recent_blocks:
                    mask[m, n] = 1
        return mask, frac, margin
    o.select_blocks = f


def _mut_sink_replaces_selection(o):
    orig = o.select_blocks

    def f(mass, tau, protect_last=True, sink_blocks=0, recent_blocks=0):
        mask, frac, margin = orig(mass, tau, protect_last, sink_blocks, recent_blocks)
        if sink_blocks:
            mask[:, sink_blocks:] = np.triu(np.tril(mask), 0)[:, sink_blocks:] * 0 + mask[:, sink_blocks:] * (recent_blocks > 0)
        return mask, frac, margin
    o.select_blocks = f


def _mut_attention_strict_causal(o):
    orig = o.attention_row_block

    def f(Qh, Kg, Vg, mask_row, m, B):
        # shifts the causal boundary by one: token i no longer sees itself
        out, lse = orig(Qh, np.roll(Kg, 1, axis=0), np.roll(Vg, 1, axis=0), mask_row, m, B)
        return out, lse
    o.attention_row_block = f


def _mut_attention_wrong_kv_head(o):
    orig = o.sparse_attention

    def f(Q, K, V, mask, B, rows=None):
        Hkv = K.shape[0]
        perm = [(g + 1) % Hkv for g in range(Hkv)]
        return orig(Q, K[perm], V[perm], mask, B, rows)
    o.sparse_attention = f


def _mut_key_set_strict(o):
    def f(a_row, tau):
        order = np.argsort(-a_row, kind="stable")
        cum = np.cumsum(a_row[order])
        reached = np.nonzero(cum > tau)[0]
        k = int(reached[0]) + 1 if reached.size else a_row.shape[0]
        keep = np.zeros(a_row.shape[0], dtype=bool)
        keep[order[:k]] = True
        return keep
    o.important_key_set = f


def _mut_accuracy_ignores_causality(o):
    def f(Qh, Kg, mask_row, i, B, tau):
        star = o.important_key_set(o.attention_row(Qh, Kg, i), tau)
        pred = np.repeat(mask_row.astype(bool), B)           # whole blocks, also positions after i
        inter = int((pred[: i + 1] & star).sum())
        return inter, int(pred.sum()), int(star.sum())
    o.selection_accuracy_query = f


def _mut_accuracy_swaps_precision_recall(o):
    orig = o.selection_accuracy_query

    def f(*a):
        inter, pred, star = orig(*a)
        return inter, star, pred
    o.selection_accuracy_query = f


def _mut_packed_mask_leaks_into_previous_sequence(o):
    def f(Hq, blocks):
        Nb = sum(blocks)
        return np.broadcast_to(np.tril(np.ones((Nb, Nb), dtype=np.uint8)), (Hq, Nb, Nb)).copy()
    o.packed_causal_block_mask = f


def _mut_packed_ranges_off_by_one(o):
    def f(blocks):
        out, at = [], 0
        for nb in blocks:
            out.append((at, at + nb))
            at += nb
        return out[:-1] + [(out[-1][0] - 1, out[-1][1])] if len(out) > 1 else out
    o.sequence_block_ranges = f


def _mut_token_diagonal_excludes_own_key(o):
    orig = o.stride_scores

    def f(Qh, Kg, S, h, mode="head", layer=0, diagonal="stride"):
        I = orig(Qh, Kg, S, h, mode, layer, "stride")
        if diagonal == "token":
            L, d = Qh.shape
            pos = o.sample_positions(L, S, h, mode, layer)
            for i in range(L // S):
                I[i, i] = Qh[pos[i]].astype(np.float64) @ Kg[i * S: pos[i]].astype(np.float64).sum(axis=0) / (S * math.sqrt(d))
        return I
    o.stride_scores = f


def _mut_token_diagonal_ignored(o):
    orig = o.stride_scores
    o.stride_scores = lambda Qh, Kg, S, h, mode="head", layer=0, diagonal="stride": orig(Qh, Kg, S, h, mode, layer, "stride")


def _mut_ragged_drops_partial_block(o):
    orig = o.block_mass
    o.block_mass = lambda P, R, Nb=None: orig(P[: P.shape[0] // R * R, : P.shape[0] // R * R], R, Nb)


def _mut_ragged_attention_reads_past_partial_block(o):
    orig = o.attention_row_block

    def f(Qh, Kg, Vg, mask_row, m, B):
        L = Qh.shape[0]
        if (m + 1) * B > L:                       # treats the partial block as if the previous full block ended the row
            mask_row = mask_row.copy()
            mask_row[m] = 0
        return orig(Qh, Kg, Vg, mask_row, m, B)
    o.attention_row_block = f


def _mut_packed_partial_block_not_protected(o):
    """The last sequence's partial last block is treated as an ordinary row (protection applied one block early)."""
    orig = o.estimate_packed

    def f(Q, K, S, B, tau, blocks, protect_last=True, *a, **kw):
        mask, frac, margin = orig(Q, K, S, B, tau, blocks, protect_last, *a, **kw)
        L = Q.shape[1]
        if L % B and protect_last:
            plain = orig(Q, K, S, B, tau, blocks, False, *a, **kw)[0]
            mask[:, -1] = plain[:, -1]
        return mask, frac, margin
    o.estimate_packed = f


def _mut_step_uses_queries_before_the_step(o):
    """The step's first row is estimated from every sampled position of its block, also those before q0."""
    def f(Qh, Kg, h, q0, S, B, tau, *a, **kw):
        mask, frac, margin = o.estimate_head(Qh, Kg, h, S, B, tau, *a, **kw)
        return mask[q0 // B:], frac[q0 // B:], margin[q0 // B:]
    o.estimate_step_head = f


def _mut_step_empty_row_selects_nothing(o):
    """A row of the step without a sampled query selects no block instead of all of them."""
    orig = o.estimate_step_head

    def f(Qh, Kg, h, q0, S, B, tau, *a, **kw):
        mask, frac, margin = orig(Qh, Kg, h, q0, S, B, tau, *a, **kw)
        for r in range(mask.shape[0]):
            if not frac[r].any():
                mask[r] = 0
        return mask, frac, margin
    o.estimate_step_head = f


MUTANTS = [_mut_step_uses_queries_before_the_step, _mut_step_empty_row_selects_nothing, _mut_packed_partial_block_not_protected, _mut_ragged_drops_partial_block, _mut_ragged_attention_reads_past_partial_block, _mut_packed_mask_leaks_into_previous_sequence, _mut_token_diagonal_excludes_own_key, _mut_token_diagonal_ignored, _mut_packed_ranges_off_by_one,
    _mut_offset_ascending, _mut_offset_ignores_head, _mut_key_window_shifted, _mut_missing_one_over_S,
    _mut_missing_sqrt_d, _mut_noncausal_softmax, _mut_block_mass_transposed, _mut_strict_threshold,
    _mut_unnormalised_threshold, _mut_ties_larger_index_first, _mut_no_protection,
    _mut_attention_strict_causal, _mut_attention_wrong_kv_head,
    _mut_key_set_strict, _mut_accuracy_ignores_causality, _mut_accuracy_swaps_precision_recall,
    _mut_hybrid_ignores_layer, _mut_layer_mode_uses_head, _mut_recent_excludes_diagonal, _mut_sink_replaces_selection,
]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda f: f.__name__)
def test_planted_mistake_is_caught(mutant):
    """Each plausible mistake, planted in a private copy of the oracle, must fail at least one pin."""
    mod = _fresh_copy()
    mutant(mod)
    failed = []
    for pin in pins.ALL_PINS:
        try:
            pin(mod)
        except AssertionError:
            failed.append(pin.__name__)
        # any other exception propagates: a mutant that crashes instead of computing a wrong value has rotted
        # (its signature no longer matches the oracle's) and must be repaired, not counted as caught
    assert failed, f"{mutant.__name__} slipped through every pin"


def test_compare_masks_rule():
    ref = np.zeros((1, 3, 3), dtype=np.uint8)
    ref[0, 2] = [1, 1, 0]
    margin = np.full((1, 3, 3), 0.3)
    frac = np.zeros((1, 3, 3))
    frac[0, 2] = [0.5, 0.3, 0.2]
    test = ref.copy()
    assert rr_oracle.compare_masks(ref, margin, frac, test)["mismatch"] == 0
    test[0, 2, 2] = 1
    r = rr_oracle.compare_masks(ref, margin, frac, test)
    assert r == {"mismatch": 1, "excused": 0, "near_tie_rows": 0, "failed": 1}
    margin[0, 2, 2] = 5e-5
    r = rr_oracle.compare_masks(ref, margin, frac, test)
    assert r["excused"] == 1 and r["failed"] == 0
    # swap of two equally heavy blocks at the cut
    margin[:] = 0.3
    frac[0, 2] = [0.5, 0.25, 0.25 + 1e-9]
    test = ref.copy()
    test[0, 2, 1], test[0, 2, 2] = 0, 1
    r = rr_oracle.compare_masks(ref, margin, frac, test)
    # counted for information, but only the margin rule excuses a block
    assert r["near_tie_rows"] == 1 and r["failed"] == 2
