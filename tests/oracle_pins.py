"""Pins for the CPU oracle: each function checks the oracle module it is given against
something the oracle did not produce (a library routine, a closed form, an invariant, the
paper's rule worked by hand, brute force).  They take the module as an argument so that the
mutation test can hand them a deliberately broken copy and see them fail.
"""
from __future__ import annotations

import itertools
import math
import os
from fractions import Fraction

import numpy as np
import torch

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _library_causal_attention(Q, K, V):
    """torch's fp64 scaled_dot_product_attention with the KV heads repeated (independent of the oracle)."""
    G = Q.shape[0] // K.shape[0]
    q = torch.from_numpy(Q).double()[None]
    k = torch.from_numpy(K).double().repeat_interleave(G, dim=0)[None]
    v = torch.from_numpy(V).double().repeat_interleave(G, dim=0)[None]
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0].numpy()


def _library_causal_probs(q, k):
    """softmax(q k^T / sqrt(d)) with the strictly upper triangle removed, by torch.softmax."""
    logits = torch.from_numpy(q).double() @ torch.from_numpy(k).double().T / math.sqrt(q.shape[1])
    n = logits.shape[0]
    logits = logits.masked_fill(torch.triu(torch.ones(n, n, dtype=torch.bool), 1), float("-inf"))
    return torch.softmax(logits, dim=1).numpy()


# ------------------------------------------------------------------ Sec. 3.1

def pin_sampling_golden(o):
    rows = [list(map(int, l.split())) for l in open(os.path.join(GOLDEN, "sampling_offsets_S4.txt"))
            if l.strip() and not l.startswith("#")]
    for h, off, p0, p1, p2 in rows:
        pos = o.sample_positions(12, 4, h)
        assert pos.tolist() == [p0, p1, p2], (h, pos)
        assert all(4 * i <= p < 4 * (i + 1) for i, p in enumerate(pos))
        assert pos[0] == off
    # all offsets of a stride are covered exactly when there are at least S heads
    for S, H in [(4, 3), (4, 4), (8, 4), (8, 8), (16, 32)]:
        offs = {int(o.sample_positions(S, S, h)[0]) for h in range(H)}
        assert (offs == set(range(S))) == (H >= S)


def pin_offset_modes_golden(o):
    """Ablation offsets (Sec. 4, round-robin strategies; reading R8), worked by hand for S = 4, layer 3."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "offset_modes_S4_layer3.txt"))
            if l.strip() and not l.startswith("#")]
    for mode, h, off in rows:
        pos = o.sample_positions(12, 4, int(h), mode, 3)
        assert pos.tolist() == [int(off), 4 + int(off), 8 + int(off)], (mode, h, pos)
    # layer 0 makes "hybrid" the head rule and "layer" the fixed rule
    for h in range(9):
        assert np.array_equal(o.sample_positions(40, 8, h, "hybrid", 0), o.sample_positions(40, 8, h))
        assert np.array_equal(o.sample_positions(40, 8, h, "layer", 0), o.sample_positions(40, 8, h, "fixed"))
    # whatever the mode, only the sampled rows of Q may matter
    L, d, S, B, Hq, Hkv = 64, 8, 4, 16, 6, 2
    Q, K = _rand((Hq, L, d), 21), _rand((Hkv, L, d), 22)
    for mode, layer in (("fixed", 0), ("layer", 5), ("hybrid", 2)):
        ref = o.estimate(Q, K, S, B, 0.8, True, mode, layer)
        Qp = np.full_like(Q, np.nan)
        for h in range(Hq):
            phase = {"fixed": 0, "layer": layer, "hybrid": h + layer}[mode]
            off = S - 1 - (phase % S)
            Qp[h, off::S] = Q[h, off::S]
        got = o.estimate(Qp, K, S, B, 0.8, True, mode, layer)
        assert np.isfinite(got[1]).all() and np.array_equal(ref[0], got[0])


def pin_sink_recent_is_a_union(o):
    """Sink / recent protection (reading R8) only adds blocks: the result is Top-tau OR the forced set."""
    L, d, S, B, Hq, Hkv = 96, 8, 2, 8, 2, 1
    Q, K = _rand((Hq, L, d), 23), _rand((Hkv, L, d), 24)
    Nb = L // B
    base = o.estimate(Q, K, S, B, 0.5, False)[0]
    m, n = np.arange(Nb)[:, None], np.arange(Nb)[None, :]
    for sink, recent in ((0, 0), (1, 0), (0, 1), (2, 3), (Nb, 0), (0, Nb)):
        got = o.estimate(Q, K, S, B, 0.5, False, "head", 0, sink, recent)[0]
        forced = ((n < sink) | (n > m - recent)) & (n <= m)
        assert np.array_equal(got.astype(bool), base.astype(bool) | forced[None]), (sink, recent)
    assert o.estimate(Q, K, S, B, 0.5, False, "head", 0, 0, 1)[0][:, np.arange(Nb), np.arange(Nb)].all()


def pin_important_key_set_bruteforce(o):
    """Appendix, first equation: the set is a smallest one reaching tau -- enumerate all subsets."""
    import itertools
    rng = np.random.default_rng(31)
    for n in (1, 2, 5, 9):
        for tau in (0.3, 0.8, 0.95, 1.0):
            a = rng.random(n) ** 3
            a /= a.sum()
            keep = o.important_key_set(a, tau)
            assert a[keep].sum() >= min(tau, a.sum()) - 1e-15
            best = min(k for k in range(1, n + 1)
                       for c in itertools.combinations(range(n), k) if a[list(c)].sum() >= tau - 1e-15)
            assert keep.sum() == best, (n, tau)
    # equal values: smaller positions first
    assert o.important_key_set(np.full(8, 0.125), 0.5).tolist() == [True] * 4 + [False] * 4


def pin_selection_accuracy_closed_forms(o):
    """Appendix, precision / recall equations on cases with closed forms."""
    L, d, B, Hq = 32, 8, 8, 2
    Nb = L // B
    tau = 0.73        # tau (i+1) is never an integer for i < 32: no decision sits on a rounding boundary
    # zero queries: every causal row is exactly uniform, A_ij = 1/(i+1), K*_i = first ceil(tau (i+1)) positions
    Q = np.zeros((Hq, L, d))
    K = _rand((1, L, d), 33)
    full = np.tril(np.ones((Nb, Nb), dtype=np.uint8))[None].repeat(Hq, 0)
    acc = o.selection_accuracy(Q, K, full, B, tau)
    star = [math.ceil(tau * (i + 1) - 1e-12) for i in range(L)]
    want_p = sum(s / (i + 1) for i, s in enumerate(star)) / L      # predicted set = all i+1 causal positions
    assert np.allclose(acc[:, 0], want_p) and np.allclose(acc[:, 1], 1.0)
    assert np.allclose(acc[:, 2], 2 * want_p / (want_p + 1))
    # only the first block selected: predicted set = positions 0 .. min(i, B-1), all inside K* while
    # ceil(tau (i+1)) >= min(i+1, B)
    first = np.zeros_like(full)
    first[:, :, 0] = 1
    acc = o.selection_accuracy(Q, K, first, B, tau)
    inter = [min(min(i + 1, B), s) for i, s in enumerate(star)]
    want_p = sum(x / min(i + 1, B) for i, x in enumerate(inter)) / L
    want_r = sum(x / s for x, s in zip(inter, star)) / L
    assert np.allclose(acc[:, 0], want_p) and np.allclose(acc[:, 1], want_r)
    # one dominant key per query (a huge logit on key i): K*_i = {i}; diagonal-only mask has recall 1
    Q2 = np.zeros((1, L, L))
    K2 = np.zeros((1, L, L))
    for i in range(L):
        Q2[0, i, i] = 40.0
        K2[0, i, i] = 40.0
    diag = np.eye(Nb, dtype=np.uint8)[None]
    acc = o.selection_accuracy(Q2, K2, diag, B, 0.9)
    want_p = sum(1.0 / ((i % B) + 1) for i in range(L)) / L        # predicted set = the diagonal block up to i
    assert np.allclose(acc[0, 1], 1.0) and np.allclose(acc[0, 0], want_p)
    # sampling every 4th position averages exactly those queries
    a4 = o.selection_accuracy(Q2, K2, diag, B, 0.9, step=4)
    assert np.allclose(a4[0, 0], sum(1.0 / ((i % B) + 1) for i in range(3, L, 4)) / (L // 4))


def pin_unsampled_queries_unused(o):
    """Only rows i*S + S-1-(h mod S) of Q may influence the estimate: poison every other row."""
    L, d, S, B, Hq, Hkv = 64, 8, 4, 16, 6, 2
    Q = _rand((Hq, L, d), 1)
    K = _rand((Hkv, L, d), 2)
    ref = o.estimate(Q, K, S, B, 0.8)
    Qp = np.full_like(Q, np.nan)
    for h in range(Hq):
        off = S - 1 - (h % S)
        Qp[h, off::S] = Q[h, off::S]
    got = o.estimate(Qp, K, S, B, 0.8)
    assert np.isfinite(got[1]).all()
    assert np.array_equal(ref[0], got[0]) and np.allclose(ref[1], got[1], rtol=0, atol=0)


def pin_gqa_head_mapping(o):
    """Query head h reads KV head h // G: blank all other KV heads with NaN, one head at a time."""
    L, d, S, B, Hq, Hkv = 32, 8, 2, 8, 6, 3
    Q, K, V = _rand((Hq, L, d), 3), _rand((Hkv, L, d), 4), _rand((Hkv, L, d), 5)
    G = Hq // Hkv
    full_mask, full_frac, _ = o.estimate(Q, K, S, B, 0.7)
    full_O, _ = o.sparse_attention(Q, K, V, full_mask, B)
    for h in range(Hq):
        Kp, Vp = np.full_like(K, np.nan), np.full_like(V, np.nan)
        Kp[h // G], Vp[h // G] = K[h // G], V[h // G]
        m, f, _ = o.estimate_head(Q[h], Kp[h // G], h, S, B, 0.7)
        assert np.array_equal(m, full_mask[h]) and np.array_equal(f, full_frac[h])
        res = o.sparse_attention(Q, Kp, Vp, full_mask, B, rows=[(h, 1), (h, L // B - 1)])
        for (hh, mm), (ob, _l) in res.items():
            assert np.array_equal(ob, full_O[hh, mm * B:(mm + 1) * B])


# ------------------------------------------------------------------ Sec. 3.2 / 3.3 (mass)

def pin_stride1_is_exact_block_mass(o):
    """S = 1: every head samples every query, the stride sum is the key itself, so the stride-level
    softmax is the exact causal attention matrix and the block mass its block sums."""
    L, d, B = 48, 8, 8
    Hq, Hkv = 4, 2
    Q, K = _rand((Hq, L, d), 6), _rand((Hkv, L, d), 7)
    Nb = L // B
    for h in range(Hq):
        A = _library_causal_probs(Q[h], K[h // 2])
        P = o.stride_softmax(o.stride_scores(Q[h], K[h // 2], 1, h))
        assert np.allclose(P, A, atol=1e-13)
        mass = o.block_mass(P, B)
        for m in range(Nb):
            for n in range(Nb):
                want = sum(A[i, j] for i in range(m * B, (m + 1) * B) for j in range(n * B, (n + 1) * B))
                assert abs(mass[m, n] - want) < 1e-12, (m, n)


def pin_stride_constant_keys(o):
    """Keys equal inside each stride (plus a perturbation that sums to zero inside the stride):
    the mean key of a stride is that common key, so I[i, j] is the ordinary scaled logit between
    the sampled query and the representative key, and P is a library causal softmax of those."""
    L, d, S = 60, 8, 5
    Ls = L // S
    rep = _rand((Ls, d), 8)
    delta = _rand((Ls, S, d), 9)
    delta -= delta.mean(axis=1, keepdims=True)
    Kg = (rep[:, None, :] + delta).reshape(L, d)
    Qh = _rand((L, d), 10)
    for h in (0, 1, 3, 4, 7):
        off = S - 1 - (h % S)
        A = _library_causal_probs(Qh[off::S], rep)
        P = o.stride_softmax(o.stride_scores(Qh, Kg, S, h))
        assert np.allclose(P, A, atol=1e-12), h


def pin_identical_keys_closed_form(o):
    """All keys identical: row i of the causal stride softmax is uniform over its i+1 strides, so
    S[m, n] = sum_{i in block m} |{j in block n : j <= i}| / (i + 1), evaluated in rationals."""
    L, d, S, B = 96, 8, 4, 16
    R, Ls, Nb = B // S, L // S, L // B
    Kg = np.tile(_rand((1, d), 11), (L, 1))
    Qh = _rand((L, d), 12)
    P = o.stride_softmax(o.stride_scores(Qh, Kg, S, 2))
    mass = o.block_mass(P, R)
    for m in range(Nb):
        for n in range(Nb):
            want = Fraction(0)
            for i in range(m * R, (m + 1) * R):
                cnt = sum(1 for j in range(n * R, (n + 1) * R) if j <= i)
                want += Fraction(cnt, i + 1)
            assert abs(mass[m, n] - float(want)) < 1e-13, (m, n)
    # normalised fractions, zero above the diagonal, rows of block mass sum to R
    mask, frac, _ = o.select_blocks(mass, 0.9)
    assert np.allclose(mass.sum(axis=1), R, atol=1e-12)
    assert np.allclose(frac.sum(axis=1), 1.0, atol=1e-13)
    assert (np.triu(mass, 1) == 0).all() and (np.triu(mask, 1) == 0).all()


def pin_mass_invariants_random(o):
    L, d, S, B = 128, 16, 4, 16
    Q, K = _rand((3, L, d), 13) * 2.0, _rand((1, L, d), 14) * 2.0
    for h in range(3):
        P = o.stride_softmax(o.stride_scores(Q[h], K[0], S, h))
        assert np.allclose(P.sum(axis=1), 1.0, atol=1e-13)
        assert (np.triu(P, 1) == 0).all()
        mass = o.block_mass(P, B // S)
        assert np.allclose(mass.sum(axis=1), B // S, atol=1e-12)
        assert (np.triu(mass, 1) == 0).all()


# ------------------------------------------------------------------ Sec. 3.3 (selection)

def pin_top_tau_bruteforce(o):
    """The selected set has the smallest cardinality that reaches tau, and among the sets of that
    cardinality it has the largest mass (the minimal-set notion of the appendix on selection accuracy)."""
    rng = np.random.default_rng(15)
    for trial in range(60):
        n = int(rng.integers(1, 11))
        mass = rng.random(n) ** 3 + 1e-3
        tau = float(rng.choice([0.3, 0.5, 0.8, 0.9, 0.95, 0.999]))
        sel, order, cum = o.top_tau_row(mass, tau)
        total = math.fsum(mass)
        got = math.fsum(mass[sel])
        assert got >= tau * total - 1e-15
        k = int(sel.sum())
        best_k, best_mass = None, None
        for size in range(1, n + 1):
            best = max(math.fsum(mass[list(c)]) for c in itertools.combinations(range(n), size))
            if best >= tau * total - 1e-15:
                best_k, best_mass = size, best
                break
        assert k == best_k, (trial, k, best_k)
        assert abs(got - best_mass) < 1e-14
        # minimality: without its lightest member the set falls below tau
        if k > 1:
            assert got - mass[sel].min() < tau * total


def pin_top_tau_ties_and_threshold(o):
    sel, order, _ = o.top_tau_row(np.array([0.25, 0.25, 0.25, 0.25]), 0.5)
    assert sel.tolist() == [True, True, False, False]           # equal masses: smaller index first
    assert order.tolist() == [0, 1, 2, 3]
    sel, _, _ = o.top_tau_row(np.array([0.25, 0.5, 0.25]), 0.5)
    assert sel.tolist() == [False, True, False]                 # cumulative == tau suffices (>=)
    sel, _, _ = o.top_tau_row(np.array([1.0, 2.0, 4.0, 1.0]), 0.75)
    assert sel.tolist() == [False, True, True, False]           # compared against tau * row total
    sel, _, _ = o.top_tau_row(np.array([0.1, 0.2, 0.3]), 1.0)
    assert sel.all()                                            # tau = 1 keeps every candidate
    mass = np.tril(np.ones((4, 4))) * np.array([4.0, 3.0, 2.0, 1.0])[None, :]
    mask, frac, margin = o.select_blocks(mass, 0.5, protect_last=True)
    assert mask[3].tolist() == [1, 1, 1, 1]                     # protected last query block
    assert mask[2].tolist() == [1, 1, 0, 0]                     # 4/9 < 0.5 <= 7/9
    mask2, _, _ = o.select_blocks(mass, 0.5, protect_last=False)
    assert mask2[3].tolist() == [1, 1, 0, 0] and np.array_equal(mask2[:3], mask[:3])
    # margins: block ranked r is selected iff the cumulative mass before it is < tau
    assert abs(margin[2, 0] - 0.5) < 1e-15 and abs(margin[2, 1] - abs(4 / 9 - 0.5)) < 1e-15
    assert abs(margin[2, 2] - abs(7 / 9 - 0.5)) < 1e-15


# ------------------------------------------------------------------ Sec. 2.1 (attention)

def pin_dense_matches_library(o):
    L, d, B = 64, 16, 16
    Q, K, V = _rand((4, L, d), 16) * 1.5, _rand((2, L, d), 17) * 1.5, _rand((2, L, d), 18)
    want = _library_causal_attention(Q, K, V)
    O, lse = o.dense_attention(Q, K, V, B)
    assert np.allclose(O, want, atol=1e-12)
    for h in range(4):
        logits = torch.from_numpy(Q[h]) @ torch.from_numpy(K[h // 2]).T / math.sqrt(d)
        logits = logits.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
        assert np.allclose(lse[h], torch.logsumexp(logits, dim=1).numpy(), atol=1e-12)


def pin_tau_one_is_dense(o):
    L, d, S, B = 64, 16, 4, 16
    Q, K, V = _rand((4, L, d), 19), _rand((2, L, d), 20), _rand((2, L, d), 21)
    mask, _, _ = o.estimate(Q, K, S, B, 1.0)
    assert np.array_equal(mask, np.broadcast_to(np.tril(np.ones((4, 4), dtype=np.uint8)), (4, 4, 4)))
    O, _ = o.sparse_attention(Q, K, V, mask, B)
    assert np.allclose(O, _library_causal_attention(Q, K, V), atol=1e-12)


def pin_sparse_matches_library_with_mask(o):
    """A random block mask: compare with torch's attention given the expanded token mask."""
    L, d, B = 64, 8, 16
    Nb = L // B
    rng = np.random.default_rng(22)
    Q, K, V = _rand((2, L, d), 23), _rand((1, L, d), 24), _rand((1, L, d), 25)
    mask = (rng.random((2, Nb, Nb)) < 0.5).astype(np.uint8)
    mask[:, np.arange(Nb), np.arange(Nb)] = 1
    mask[0, 2, 2] = 0                      # a row that omits its diagonal block is legal
    mask[0, 2, 0] = 1
    mask *= np.tril(np.ones((Nb, Nb), dtype=np.uint8))
    O, _ = o.sparse_attention(Q, K, V, mask, B)
    tok = np.kron(mask, np.ones((B, B), dtype=np.uint8)).astype(bool) & np.tril(np.ones((L, L), dtype=bool))
    q = torch.from_numpy(Q)[None]
    k = torch.from_numpy(K).repeat_interleave(2, dim=0)[None]
    v = torch.from_numpy(V).repeat_interleave(2, dim=0)[None]
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=torch.from_numpy(tok)[None])[0]
    assert np.allclose(O, want.numpy(), atol=1e-12)


def pin_constant_values_and_empty_rows(o):
    L, d, B = 32, 8, 8
    Nb = L // B
    Q, K = _rand((2, L, d), 26), _rand((2, L, d), 27)
    V = np.tile(np.arange(d, dtype=np.float64)[None, None, :], (2, L, 1))
    mask = np.tril((np.random.default_rng(28).random((2, Nb, Nb)) < 0.6)).astype(np.uint8)
    mask[:, np.arange(Nb), np.arange(Nb)] = 1
    mask[1, 2, :] = 0                      # a query block with nothing selected
    O, lse = o.sparse_attention(Q, K, V, mask, B)
    for h in range(2):
        for m in range(Nb):
            blk = O[h, m * B:(m + 1) * B]
            if mask[h, m].any():
                assert np.allclose(blk, np.arange(d)[None, :], atol=1e-12)
            else:
                assert (blk == 0).all() and np.isneginf(lse[h, m * B:(m + 1) * B]).all()


def pin_packed_sequences_are_independent(o):
    """Packed batch (reading R10): block-diagonal masks on the packed tensors give, sequence by sequence,
    what a library attention gives for that sequence alone; estimation of a packed batch is the
    per-sequence estimation, unmoved by the other sequences' contents."""
    d, S, B = 8, 2, 8
    blocks = [3, 1, 4]
    L = B * sum(blocks)
    Q, K, V = _rand((4, L, d), 61) * 1.5, _rand((2, L, d), 62) * 1.5, _rand((2, L, d), 63)
    ranges = o.sequence_block_ranges(blocks)
    assert ranges == [(0, 3), (3, 4), (4, 8)]
    # dense baseline of the packed batch == library attention per sequence
    O, _ = o.sparse_attention(Q, K, V, o.packed_causal_block_mask(4, blocks), B)
    for (b0, b1) in ranges:
        sl = slice(b0 * B, b1 * B)
        assert np.allclose(O[:, sl], _library_causal_attention(Q[:, sl], K[:, sl], V[:, sl]), atol=1e-12)
    # estimation: equals the single-sequence estimation of each slice, also with the other slices poisoned
    mask, frac, _ = o.estimate_packed(Q, K, S, B, 0.7, blocks, sink_blocks=1)
    for (b0, b1) in ranges:
        sl = slice(b0 * B, b1 * B)
        Kp, Qp = np.full_like(K, np.nan), np.full_like(Q, np.nan)
        Kp[:, sl], Qp[:, sl] = K[:, sl], Q[:, sl]
        mk, fr, _ = o.estimate(Qp[:, sl], Kp[:, sl], S, B, 0.7, sink_blocks=1)
        assert np.array_equal(mask[:, b0:b1, b0:b1], mk) and np.allclose(frac[:, b0:b1, b0:b1], fr, atol=0)
        assert not mask[:, b0:b1, :b0].any() and not mask[:, b0:b1, b1:].any()
        assert mask[:, b1 - 1, b0:b1].all()             # each sequence's last query block is protected
        assert mask[:, b0:b1, b0].all()                 # the sink block is the sequence's first block
    # a sparse packed mask: same outputs as attention of each slice under its own sub-mask
    O2, _ = o.sparse_attention(Q, K, V, mask, B)
    for (b0, b1) in ranges:
        sl = slice(b0 * B, b1 * B)
        want, _ = o.sparse_attention(Q[:, sl], K[:, sl], V[:, sl], mask[:, b0:b1, b0:b1], B)
        assert np.allclose(O2[:, sl], want, atol=1e-12)


def pin_packed_last_sequence_may_end_inside_a_block(o):
    """Packed batch whose LAST sequence is not a whole number of blocks (readings R7 + R10): every sequence's
    rows are those of the single-sequence estimate of that slice; the positions of the last sequence that
    follow its last complete stride are never read; its partial last block is a protected last query block."""
    d, S, B = 6, 4, 8
    blocks = [2, 3]                               # second sequence: 2 whole blocks + 5 positions (1 stride + 1 token)
    L = B * sum(blocks) - 3
    Q, K = _rand((4, L, d), 65) * 1.5, _rand((2, L, d), 66) * 1.5
    mask, frac, margin = o.estimate_packed(Q, K, S, B, 0.6, blocks)
    assert mask.shape == (4, 5, 5)
    first = o.estimate(Q[:, : 2 * B], K[:, : 2 * B], S, B, 0.6)
    last = o.estimate(Q[:, 2 * B:], K[:, 2 * B:], S, B, 0.6)
    assert last[0].shape == (4, 3, 3)
    for (b0, b1), (mk, fr, mg) in (((0, 2), first), ((2, 5), last)):
        assert np.array_equal(mask[:, b0:b1, b0:b1], mk) and np.array_equal(frac[:, b0:b1, b0:b1], fr)
        assert np.array_equal(margin[:, b0:b1, b0:b1], mg)
    assert not mask[:, 2:, :2].any() and not mask[:, :2, 2:].any()
    assert mask[:, 4, 2:5].all() and mask[:, 1, 0:2].all()          # both sequences' last query blocks are protected
    # without protection the partial block's row comes from its single complete stride: written out by hand
    m2, f2, _ = o.estimate_packed(Q, K, S, B, 0.6, blocks, protect_last=False)
    for h in range(4):
        Qs, Ks = Q[h, 2 * B:], K[h // 2, 2 * B:]
        i = 4                                                         # the stride of the partial block (local index)
        q = Qs[i * S + (S - 1 - h % S)]
        logits = np.array([q @ Ks[j * S:(j + 1) * S].sum(axis=0) for j in range(i + 1)]) / (S * math.sqrt(d))
        p = _library_causal_probs_row(logits)
        want = np.array([p[0:2].sum(), p[2:4].sum(), p[4:5].sum()])
        assert np.allclose(f2[h, 4, 2:5], want / want.sum(), atol=1e-13)
    # the token after the last complete stride is in no stride: poisoned, nothing changes
    Qp, Kp = Q.copy(), K.copy()
    Qp[:, L - 1:], Kp[:, L - 1:] = np.nan, np.nan
    mp, fp, _ = o.estimate_packed(Qp, Kp, S, B, 0.6, blocks, protect_last=False)
    assert np.array_equal(mp, m2) and np.array_equal(fp, f2)


def pin_decode_step_reductions(o):
    """Reading R12 (a step of the last Lq positions at any offset): q0 = 0 is the method; a step that starts
    at a block boundary gives the rows of the full estimate; rows of blocks that lie wholly inside the step
    are the full estimate's rows; the first, partly covered row is written out with explicit loops over the
    sampled positions the step holds; nothing before q0 is read; a one-token step that is no sampled position
    keeps every causal block (dense decoding); one that is, ranks the blocks by that single query; tau = 1
    keeps everything."""
    L, d, S, B = 61, 6, 2, 8                       # 30 strides, 8 blocks (the last holds 5 positions: 2 strides)
    R, Nb, Ls = B // S, 8, 30
    Q, K = _rand((4, L, d), 101) * 2.0, _rand((2, L, d), 102) * 2.0
    full = o.estimate(Q, K, S, B, 0.7, False)
    for q0 in (0, 16, 40):                         # block boundaries
        got = o.estimate_step(Q, K, q0, S, B, 0.7, False)
        for a, b in zip(got, full):
            assert np.array_equal(a, b[:, q0 // B:])
    for q0 in (19, 37, 58):
        Qp = Q.copy()
        Qp[:, :q0] = np.nan                        # the step does not hold these queries
        mask, frac, margin = o.estimate_step(Qp, K, q0, S, B, 0.7, False)
        first = q0 // B
        assert mask.shape == (4, Nb - first, Nb)
        for a, b in zip((mask, frac, margin), full):
            assert np.array_equal(a[:, 1:], b[:, first + 1:])       # rows wholly inside the step
        for h in range(4):                         # the partly covered row, by hand
            m = first
            mass = np.zeros(m + 1)
            for i in range(m * R, min((m + 1) * R, Ls)):
                p = i * S + (S - 1 - h % S)
                if p < q0:
                    continue
                logits = np.array([Q[h, p] @ K[h // 2, j * S:(j + 1) * S].sum(axis=0) for j in range(i + 1)]) / (S * math.sqrt(d))
                pr = _library_causal_probs_row(logits)
                for j in range(i + 1):
                    mass[j // R] += pr[j]
            if mass.sum() == 0.0:
                assert mask[h, 0, : m + 1].all() and not frac[h, 0].any()
            else:
                assert np.allclose(frac[h, 0, : m + 1], mass / mass.sum(), atol=1e-13)
                sel, _, _ = o.top_tau_row(mass, 0.7)
                assert np.array_equal(mask[h, 0, : m + 1], sel.astype(np.uint8))
            assert not mask[h, 0, m + 1:].any()
    # one token (L even here): position 59 is the sampled position of its stride for heads with h mod S = 0 only
    L1 = 60
    Q1, K1 = Q[:, :L1], K[:, :L1]
    mask, frac, _ = o.estimate_step(Q1, K1, L1 - 1, S, B, 0.5, False)
    assert mask.shape == (4, 1, Nb)
    for h in range(4):
        if h % S == 0:
            logits = np.array([Q1[h, 59] @ K1[h // 2, j * S:(j + 1) * S].sum(axis=0) for j in range(30)]) / (S * math.sqrt(d))
            pr = _library_causal_probs_row(logits)
            mass = pr.reshape(-1, R).sum(axis=1) if 30 % R == 0 else np.array([pr[n * R:(n + 1) * R].sum() for n in range(Nb)])
            sel, _, _ = o.top_tau_row(mass, 0.5)
            assert np.array_equal(mask[h, 0], sel.astype(np.uint8)) and np.allclose(frac[h, 0], mass, atol=1e-13)
        else:
            assert mask[h, 0].all() and not frac[h, 0].any()        # no sampled query: dense, as the paper decodes
    assert o.estimate_step(Q, K, 37, S, B, 1.0, False)[0][:, :, :].sum() == 4 * sum(m + 1 for m in range(37 // B, Nb))
    # with the last query block protected the last row is full whatever the step holds
    assert o.estimate_step(Q, K, 58, S, B, 0.5, True)[0][:, -1].all()


def pin_token_exact_diagonal(o):
    """diagonal = "token": scores written out with explicit loops; reductions to the default rule when the
    sampled query is the last position of its stride (fixed offsets) and when S = 1; keys after the sampled
    position of the diagonal stride are never read."""
    L, d, S = 24, 5, 4
    Q, K = _rand((3, L, d), 71), _rand((3, L, d), 72)
    for h in range(3):
        pos = o.sample_positions(L, S, h)
        I = o.stride_scores(Q[h], K[h], S, h, diagonal="token")
        for i in range(L // S):
            for j in range(L // S):
                last = pos[i] if j == i else j * S + S - 1
                want = sum(float(Q[h, pos[i]] @ K[h, k]) for k in range(j * S, last + 1)) / (S * math.sqrt(d))
                assert abs(I[i, j] - want) < 1e-12, (h, i, j)
    # fixed offsets sample the last position of a stride: nothing is cut
    assert np.array_equal(o.stride_scores(Q[1], K[1], S, 1, "fixed", 0, "token"),
                          o.stride_scores(Q[1], K[1], S, 1, "fixed", 0, "stride"))
    assert np.array_equal(o.stride_scores(Q[2], K[2], 1, 2, diagonal="token"), o.stride_scores(Q[2], K[2], 1, 2))
    # head 2 samples offset S-1-2 = 1: keys 2, 3 of the last stride follow the last sampled query
    Kp = K[2].copy()
    Kp[L - S + 2:] = np.nan
    assert np.isfinite(o.stride_scores(Q[2], Kp, S, 2, diagonal="token")[:, : L // S - 1]).all()
    assert np.isfinite(o.stride_scores(Q[2], Kp, S, 2, diagonal="token")[-1, -1])
    assert np.isnan(o.stride_scores(Q[2], Kp, S, 2, diagonal="stride")[-1, -1])
    # and the rule reaches the mask: some row differs on inputs where the cut keys matter
    Q2, K2 = _rand((2, 64, 8), 73) * 3.0, _rand((2, 64, 8), 74) * 3.0
    f_tok = o.estimate(Q2, K2, 8, 8, 0.9, diagonal="token")[1]
    f_str = o.estimate(Q2, K2, 8, 8, 0.9)[1]
    assert np.abs(f_tok - f_str).max() > 1e-3


def pin_estimate_row_is_a_row_of_estimate_head(o):
    """estimate_row (used where the full stride matrix cannot be held) against the pinned full computation."""
    L, d, S, B = 96, 8, 4, 16
    Q, K = _rand((3, L, d), 81) * 2.0, _rand((3, L, d), 82) * 2.0
    for h in range(3):
        for protect in (True, False):
            mask, frac, margin = o.estimate_head(Q[h], K[h], h, S, B, 0.8, protect)
            for m in range(L // B):
                mk, fr, mg = o.estimate_row(Q[h], K[h], h, m, S, B, 0.8, protect)
                assert np.array_equal(mk, mask[m, : m + 1])
                assert np.allclose(fr, frac[m, : m + 1], atol=1e-14) and np.allclose(mg, margin[m, : m + 1], atol=1e-13)


def pin_ragged_length(o):
    """L that is a multiple of neither S nor B (reading R7): ceil(L/B) blocks, floor(L/S) strides."""
    # attention: library softmax attention of the same length, dense and with a random block mask
    L, d, B = 53, 8, 16
    Nb = 4
    Q, K, V = _rand((2, L, d), 91) * 1.5, _rand((1, L, d), 92) * 1.5, _rand((1, L, d), 93)
    O, _ = o.dense_attention(Q, K, V, B)
    assert O.shape == (2, L, d)
    assert np.allclose(O, _library_causal_attention(Q, K, V), atol=1e-12)
    mask = np.tril((np.random.default_rng(94).random((2, Nb, Nb)) < 0.5)).astype(np.uint8)
    mask[:, np.arange(Nb), np.arange(Nb)] = 1
    O2, _ = o.sparse_attention(Q, K, V, mask, B)
    tok = np.kron(mask, np.ones((B, B), dtype=np.uint8)).astype(bool)[:, :L, :L] & np.tril(np.ones((L, L), dtype=bool))
    q = torch.from_numpy(Q)[None]
    k = torch.from_numpy(K).repeat_interleave(2, dim=0)[None]
    v = torch.from_numpy(V).repeat_interleave(2, dim=0)[None]
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=torch.from_numpy(tok)[None])[0]
    assert np.allclose(O2, want.numpy(), atol=1e-12)

    # estimation: block mass summed by explicit loops over the strides that exist
    L, d, S, B = 45, 6, 2, 8                      # 22 strides (token 44 in none), 6 blocks, the last with 2 strides
    R, Ls, Nb = B // S, L // S, 6
    Qe, Ke = _rand((3, L, d), 95) * 2.0, _rand((3, L, d), 96) * 2.0
    for h in range(3):
        mask_h, frac_h, _ = o.estimate_head(Qe[h], Ke[h], h, S, B, 0.75, False)
        assert mask_h.shape == (Nb, Nb)
        pos = [i * S + (S - 1 - h % S) for i in range(Ls)]
        mass = np.zeros((Nb, Nb))
        for i in range(Ls):
            logits = np.array([Qe[h, pos[i]] @ Ke[h, j * S:(j + 1) * S].sum(axis=0) for j in range(i + 1)]) / (S * math.sqrt(d))
            p = _library_causal_probs_row(logits)
            for j in range(i + 1):
                mass[i // R, j // R] += p[j]
        for m in range(Nb):
            assert np.allclose(frac_h[m, : m + 1], mass[m, : m + 1] / mass[m, : m + 1].sum(), atol=1e-13)
        # positions after the last complete stride are never read by the estimate
        Qp, Kp = Qe[h].copy(), Ke[h].copy()
        Qp[Ls * S:], Kp[Ls * S:] = np.nan, np.nan
        mask_p, frac_p, _ = o.estimate_head(Qp, Kp, h, S, B, 0.75, False)
        assert np.array_equal(mask_p, mask_h) and np.array_equal(frac_p, frac_h)
    # same rows as the computation on inputs filled up to a block boundary (the protected last row included)
    pad = Nb * B - L
    Qz = np.concatenate([Qe, np.full((3, pad, d), 7.0)], axis=1)
    Kz = np.concatenate([Ke, np.full((3, pad, d), -3.0)], axis=1)
    m_r, f_r, _ = o.estimate(Qe, Ke, S, B, 0.75)
    m_z, f_z, _ = o.estimate(Qz, Kz, S, B, 0.75)
    assert np.array_equal(m_r, m_z) and np.allclose(f_r[:, :-1], f_z[:, :-1], atol=1e-14)
    # a last block without one complete stride has no estimate and keeps every block
    m_s, f_s, _ = o.estimate(Qe[:, :41], Ke[:, :41], 8, 8, 0.5, False)      # 5 strides of 8, block 5 holds token 40 only
    assert m_s.shape == (3, 6, 6) and m_s[:, 5].all() and not f_s[:, 5].any()


def _library_causal_probs_row(logits):
    return torch.softmax(torch.from_numpy(np.asarray(logits, dtype=np.float64)), dim=0).numpy()


ALL_PINS = [pin_decode_step_reductions, pin_packed_last_sequence_may_end_inside_a_block, pin_ragged_length, pin_estimate_row_is_a_row_of_estimate_head, pin_packed_sequences_are_independent, pin_token_exact_diagonal, pin_important_key_set_bruteforce, pin_selection_accuracy_closed_forms, pin_offset_modes_golden, pin_sink_recent_is_a_union, 
    pin_sampling_golden,
    pin_unsampled_queries_unused,
    pin_gqa_head_mapping,
    pin_stride1_is_exact_block_mass,
    pin_stride_constant_keys,
    pin_identical_keys_closed_form,
    pin_mass_invariants_random,
    pin_top_tau_bruteforce,
    pin_top_tau_ties_and_threshold,
    pin_dense_matches_library,
    pin_tau_one_is_dense,
    pin_sparse_matches_library_with_mask,
    pin_constant_values_and_empty_rows,
]
