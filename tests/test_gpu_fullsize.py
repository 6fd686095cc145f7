"""GPU parity at the full workload sizes, in the launch configuration bench.py times (caller-owned
workspace, mask and output buffers; whole layer per call).

Estimation: the block mask of every head is compared with the fp64 oracle in full (the oracle needs
about a second per head at 128K).  Attention: the oracle evaluates a seeded sample of query blocks
(h, m) one by one -- always the first and the last block, the densest and the sparsest row of the
mask, plus random ones -- against the corresponding rows of the full GPU output; on top of that,
properties that hold at any size are checked on the whole output (finite everywhere; the first
token of every head attends to itself only, so its output row equals its V row).
"""
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import rr_inputs as ri
from oracle import rr_oracle as oracle
import gpu_util as gu
import oracle_rows

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


# workload, [(S, tau)], attention rows per variant, number of dense-baseline rows
FULL = {
    "cfg1": ("cfg1", [(16, 0.9), (16, 0.95)], [2048, 512], 64),
    "cfg2": ("cfg2", [(16, 0.9), (16, 0.95)], [512, 512], 24),
    "cfg3": ("cfg3", [(16, 0.9), (8, 0.9)], [512, 512], 24),
    "cfg4": ("cfg4", [(16, 0.9)], [512], 24),
}


def _sample_rows(dense, n_rows, seed):
    """(h, m) pairs: of EVERY head the first block, its densest row and its sparsest row (relative to the causal
    length, lower half of the sequence); the last block of four heads; seeded random ones up to n_rows."""
    H, Nb, _ = dense.shape
    rng = np.random.default_rng(seed)
    cnt = dense.sum(-1).astype(np.int64)
    rows = set()
    rel = cnt[:, Nb // 2:] / np.arange(Nb // 2 + 1, Nb + 1)[None, :]
    for h in range(H):
        rows.add((h, 0))
        rows.add((h, int(np.argmax(cnt[h]))))
        rows.add((h, Nb // 2 + int(np.argmin(rel[h]))))
    for h in {0, H - 1, int(rng.integers(H)), int(rng.integers(H))}:
        rows.add((h, Nb - 1))
    while len(rows) < n_rows:
        rows.add((int(rng.integers(H)), int(rng.integers(Nb))))
    return sorted(rows)


def _check_rows(x, w, O, lse, mask_np, rows, label, ref_mask=None, pool_key=None):
    """GPU rows against the oracle evaluated with the GPU's mask.  With ref_mask (the oracle's own mask) the rows
    whose mask row agrees with it are at the same time the end-to-end comparison (oracle estimate -> oracle
    attention against GPU estimate -> GPU attention); the others differ by excused blocks only and are counted.
    pool_key = (workload name, cut length or 0): the oracle rows are computed by worker processes that
    regenerate that workload; without it, by threads of this process on x."""
    G = w.G
    worst_max, sum_abs, n = 0.0, 0.0, 0
    Oc = O[0].float()
    if pool_key is not None and len(rows) > 64:
        refs = oracle_rows.attention_rows(pool_key[0], pool_key[1], w.B, G, rows, mask_np,
                                          progress=lambda a, b: _say(f"[full] {label}: oracle rows {a}/{b}"))
    else:
        with ThreadPoolExecutor(8) as ex:      # numpy releases the GIL inside its BLAS calls
            refs = list(ex.map(lambda hm: oracle.attention_row_block(x["Q"][hm[0]], x["K"][hm[0] // G], x["V"][hm[0] // G],
                                                                     mask_np[hm[0], hm[1]], hm[1], w.B), rows))
    end_to_end = 0
    for (h, m), (ref_O, ref_lse) in zip(rows, refs):
        got = Oc[h, m * w.B:(m + 1) * w.B].cpu().numpy().astype(np.float64)
        diff = np.abs(got - ref_O)
        worst_max = max(worst_max, float(diff.max()))
        sum_abs += float(diff.sum())
        n += diff.size
        got_lse = lse[0, h, m * w.B:(m + 1) * w.B].cpu().numpy().astype(np.float64)
        assert np.abs(got_lse - ref_lse).max() < 2e-2, (label, h, m)
        if ref_mask is not None and np.array_equal(ref_mask[h, m], mask_np[h, m]):
            end_to_end += 1
    tail = "" if ref_mask is None else f" ({end_to_end} of them end to end: the oracle's own mask row is the same)"
    _say(f"[full] {label}: {len(rows)} query blocks{tail}, max abs {worst_max:.3e}, mean abs {sum_abs / n:.3e}")
    assert worst_max <= gu.BF16_MAX_ABS and sum_abs / n <= gu.BF16_MEAN_ABS, label
    if ref_mask is not None:
        assert end_to_end >= len(rows) - 8, label          # at most a handful of rows may hold an excused block


@pytest.mark.parametrize("name", list(FULL))
def test_full_size_path_matches_oracle(name):
    import paper_2602_05853_amd as rr
    cfg, variants, n_rows, n_dense = FULL[name]
    w = ri.get_config(cfg)
    _say(f"[full] case={name} L={w.L} Hq={w.Hq} Hkv={w.Hkv} d={w.d} {w.dtype} B={w.B}")
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    Q, K, V = t["Q"], t["K"], t["V"]
    O = torch.empty_like(Q)
    lse = torch.empty((1, w.Hq, w.L), dtype=torch.float32, device=Q.device)
    for (S, tau), nr in zip(variants, n_rows):
        _say(f"[full] {name}: estimate S={S} tau={tau}")
        ws = torch.empty(rr.rr_workspace_bytes(Q, K, S, w.B), dtype=torch.uint8, device=Q.device)
        mask = rr.BlockMask.allocate(1, w.Hq, w.Nb, w.B, Q.device, dense=True, block_mass=True, Hkv=w.Hkv)
        rr.rr_estimate(Q, K, S, w.B, tau, out=mask, workspace=ws)
        torch.cuda.synchronize()
        del ws
        ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, S, w.B, tau, True, threads=16)
        gu.check_mask_structures(mask)
        rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
        _say(f"[full] {name} S={S} tau={tau}: {rep}")
        assert rep["failed"] == 0
        assert rep["mass_max_abs_err"] < 2e-5
        del ref_frac, ref_margin

        _say(f"[full] {name}: sparse attention S={S} tau={tau}")
        O.fill_(float("nan"))
        rr.rr_sparse_attn(Q, K, V, mask, O=O, lse=lse)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(O).all())
        assert torch.equal(O[0, :, 0, :], V[0].repeat_interleave(w.G, 0)[:, 0, :])
        # every row, whatever order the workgroups start in: the same launch without the row-order hint
        # must give the same bits
        order, mask.row_order = mask.row_order, None
        O2 = rr.rr_sparse_attn(Q, K, V, mask)
        torch.cuda.synchronize()
        assert torch.equal(O2, O), "the launch order changed a result"
        del O2
        mask.row_order = order
        mask_np = mask.dense.cpu().numpy()[0]
        rows = _sample_rows(mask_np, nr, seed=w.seed + int(tau * 100) + S)
        _check_rows(x, w, O, lse, mask_np, rows, f"{name} sparse S={S} tau={tau}", ref_mask=ref_mask, pool_key=(cfg, 0))
        del mask, ref_mask

    _say(f"[full] {name}: dense baseline")
    O.fill_(float("nan"))
    rr.rr_dense_attn(Q, K, V, w.B, O=O, lse=lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all())
    rng = np.random.default_rng(w.seed)
    rows = sorted({(0, 0), (w.Hq - 1, w.Nb - 1)} | {(int(rng.integers(w.Hq)), int(rng.integers(w.Nb)))
                                                    for _ in range(n_dense)})
    causal = oracle.causal_block_mask(1, w.Nb)[0]
    _check_rows(x, w, O, lse, np.broadcast_to(causal, (w.Hq, w.Nb, w.Nb)), rows, f"{name} dense")
    # every row of the list-walking launch: with tau = 1 the estimate lists every causal block, and the sparse
    # call must then reproduce the dense call bit for bit over the whole tensor
    S = variants[0][0]
    mask = rr.rr_estimate(Q, K, S, w.B, 1.0)
    assert int(mask.row_count.sum()) == w.Hq * w.Nb * (w.Nb + 1) // 2
    O1 = rr.rr_sparse_attn(Q, K, V, mask)
    torch.cuda.synchronize()
    assert torch.equal(O1, O), "sparse attention over every causal block differs from the dense baseline"
    _say(f"[full] {name}: tau = 1 sparse == dense on all {w.Hq * w.Nb} rows")


def test_full_size_decode_steps_cfg2():
    """One and two new tokens against the 128K context of the headline workload, through the entry points with
    a workspace (the decode kernel, the launch bench.py times as decode_step): masks of the heads that hold a
    sampled position against the oracle's step estimate, every other head dense (reading R14), and all output
    rows against oracle attention rows."""
    import paper_2602_05853_amd as rr
    w = ri.get_config("cfg2")
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    K, V = t["K"], t["V"]
    L, B, S, G, Nb = w.L, w.B, w.S, w.G, w.Nb
    for T in (1, 2):
        q0 = L - T
        _say(f"[full] decode step cfg2: L={L} q0={q0} T={T}")
        Qc = t["Q"][:, :, q0:, :].contiguous()
        mask = rr.rr_estimate(Qc, K, S, B, 0.9, flags=0, block_mass=True)
        torch.cuda.synchronize()
        dense = mask.dense.cpu().numpy()[0]                       # [Hq, 1, Nb]
        assert dense.shape == (w.Hq, 1, Nb)
        # heads whose sampled position (Sec. 3.1) of a complete stride lies inside the step
        sampled = [h for h in range(w.Hq)
                   if any((p % S) == S - 1 - (h % S) and (p // S + 1) * S <= L for p in range(q0, L))]
        _say(f"[full] decode step T={T}: heads with a sampled position {sampled}")
        assert 0 < len(sampled) < w.Hq
        with ThreadPoolExecutor(4) as ex:
            refs = list(ex.map(lambda h: oracle.estimate_step_head(x["Q"][h], x["K"][h // G], h, q0, S, B, 0.9, False),
                               sampled))
        for h, (ref_mask, ref_frac, ref_margin) in zip(sampled, refs):
            rep = oracle.compare_masks(ref_mask[None], ref_margin[None], ref_frac[None], dense[h][None],
                                       margin_tol=gu.MARGIN_TOL)
            _say(f"[full] decode step T={T} head {h}: {rep}, selected {int(dense[h].sum())} of {Nb}")
            assert rep["failed"] == 0
        for h in range(w.Hq):
            if h not in sampled:
                assert int(dense[h].sum()) == Nb, h
        need = rr.rr_attn_workspace_bytes(Qc, K, B)
        assert need > 0
        wsa = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        lse_s = torch.full((1, w.Hq, T), float("nan"), dtype=torch.float32, device="cuda:0")
        lse_d = torch.full_like(lse_s, float("nan"))
        Os = torch.full_like(Qc, float("nan"))
        Od = torch.full_like(Qc, float("nan"))
        rr.rr_sparse_attn(Qc, K, V, mask, O=Os, lse=lse_s, workspace=wsa)
        rr.rr_dense_attn(Qc, K, V, B, O=Od, lse=lse_d, workspace=wsa)
        torch.cuda.synchronize()
        full_row = np.ones(Nb, dtype=np.uint8)
        with ThreadPoolExecutor(8) as ex:
            ref_s = list(ex.map(lambda h: oracle.attention_row_block(x["Q"][h], x["K"][h // G], x["V"][h // G],
                                                                     dense[h, 0], Nb - 1, B), range(w.Hq)))
            ref_d = list(ex.map(lambda h: oracle.attention_row_block(x["Q"][h], x["K"][h // G], x["V"][h // G],
                                                                     full_row, Nb - 1, B), range(w.Hq)))
        for label, got, got_lse, refs_ in (("sparse", Os, lse_s, ref_s), ("dense", Od, lse_d, ref_d)):
            assert bool(torch.isfinite(got.float()).all()) and bool(torch.isfinite(got_lse).all())
            want = np.stack([r[0][B - T:] for r in refs_])                     # the last T queries of the last block
            want_lse = np.stack([r[1][B - T:] for r in refs_])
            mx, mean = gu.attention_errors(got[0], want)
            _say(f"[full] decode step T={T} {label}: {w.Hq * T} rows, max abs {mx:.3e} mean abs {mean:.3e}")
            assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS
            assert np.abs(got_lse[0].cpu().numpy() - want_lse).max() < 2e-2


def test_long_context_256k_two_heads():
    """Twice the headline length (2048 blocks per row, 4 M block pairs per head, 64-bit offsets into the
    workspace): masks of both heads in full, three attention rows, finiteness of everything."""
    import paper_2602_05853_amd as rr
    w = ri.custom(L=262144, Hq=2, Hkv=1, d=128, dtype="bf16", B=128, S=16, seed=777, logit_gain=4.0, n_spans=64)
    _say(f"[full] case=256K L={w.L} Hq={w.Hq} Hkv={w.Hkv}")
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    mask = rr.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9, block_mass=True)
    lse = torch.empty((1, w.Hq, w.L), dtype=torch.float32, device="cuda:0")
    O = rr.rr_sparse_attn(t["Q"], t["K"], t["V"], mask, lse=lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all()) and bool(torch.isfinite(lse).all())
    ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, w.S, w.B, 0.9, True, threads=2)
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, 0.9)
    _say(f"[full] 256K: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5
    mask_np = mask.dense.cpu().numpy()[0]
    _check_rows(x, w, O, lse, mask_np, [(0, 0), (1, w.Nb - 1), (0, w.Nb // 2 + 3)], "256K sparse")


def test_full_size_packed_sequences():
    """The 128K tensors of cfg2 read as eleven packed sequences of 64K ... 128 tokens: masks of every head in
    full against the sequence-by-sequence oracle, sampled attention rows (first and last block of sequences
    included), the packed dense baseline."""
    import paper_2602_05853_amd as rr
    w = ri.get_config("cfg2")
    blocks = [512, 256, 128, 64, 32, 16, 8, 4, 2, 1, 1]
    assert sum(blocks) == w.Nb
    S, tau = 16, 0.9
    _say(f"[full] case=packed L={w.L} blocks={blocks}")
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    Q, K, V = t["Q"], t["K"], t["V"]
    sf = rr.packed_seq_first(blocks, Q.device)
    ws = torch.empty(rr.rr_workspace_bytes(Q, K, S, w.B), dtype=torch.uint8, device=Q.device)
    mask = rr.BlockMask.allocate(1, w.Hq, w.Nb, w.B, Q.device, dense=True, block_mass=True, Hkv=w.Hkv)
    rr.rr_estimate(Q, K, S, w.B, tau, out=mask, workspace=ws, seq_first=sf)
    torch.cuda.synchronize()
    del ws
    ranges = oracle.sequence_block_ranges(blocks)
    ref_mask = np.zeros((w.Hq, w.Nb, w.Nb), dtype=np.uint8)
    ref_frac = np.zeros((w.Hq, w.Nb, w.Nb), dtype=np.float64)
    ref_margin = np.full((w.Hq, w.Nb, w.Nb), np.inf, dtype=np.float64)
    for (b0, b1) in ranges:                       # estimate_packed, with the heads of a sequence in parallel
        sl = slice(b0 * w.B, b1 * w.B)
        mk, fr, mg = gu.oracle_estimate({"Q": x["Q"][:, sl], "K": x["K"][:, sl]}, S, w.B, tau, True)
        ref_mask[:, b0:b1, b0:b1], ref_frac[:, b0:b1, b0:b1], ref_margin[:, b0:b1, b0:b1] = mk, fr, mg
    gu.check_mask_structures(mask)
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
    _say(f"[full] packed: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5
    del ref_frac, ref_margin

    O = torch.full_like(Q, float("nan"))
    lse = torch.empty((1, w.Hq, w.L), dtype=torch.float32, device=Q.device)
    rr.rr_sparse_attn(Q, K, V, mask, O=O, lse=lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all())
    mask_np = mask.dense.cpu().numpy()[0]
    rng = np.random.default_rng(99)
    rows = {(int(rng.integers(w.Hq)), b0) for (b0, _) in ranges} | {(int(rng.integers(w.Hq)), b1 - 1) for (_, b1) in ranges}
    while len(rows) < 36:
        rows.add((int(rng.integers(w.Hq)), int(rng.integers(w.Nb))))
    _check_rows(x, w, O, lse, mask_np, sorted(rows), "packed sparse")

    O.fill_(float("nan"))
    rr.rr_dense_attn_packed(Q, K, V, w.B, sf, O=O, lse=lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all())
    inside = oracle.packed_causal_block_mask(1, blocks)[0]
    rows = sorted({(0, 0), (w.Hq - 1, w.Nb - 1), (3, 511), (5, 512), (7, 767), (11, 1022)})
    _check_rows(x, w, O, lse, np.broadcast_to(inside, (w.Hq, w.Nb, w.Nb)), rows, "packed dense")


def test_maximum_length_one_million_tokens():
    """The largest supported length (L/B = 8192 blocks, 65536 strides): 4 GB of softmax state behind 64-bit
    offsets, an 8192-key sort per row.  The full stride matrix is out of the oracle's reach here, so rows
    of the mask are checked one by one (first, last, around the middle, random), as are attention rows."""
    import paper_2602_05853_amd as rr
    w = ri.custom(L=1 << 20, Hq=1, Hkv=1, d=128, dtype="bf16", B=128, S=16, seed=778, logit_gain=4.0, n_spans=64)
    assert w.Nb == 8192
    _say(f"[full] case=1M L={w.L}")
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    Q, K, V = t["Q"], t["K"], t["V"]
    tau = 0.9
    mask = rr.rr_estimate(Q, K, w.S, w.B, tau, block_mass=False)
    lse = torch.empty((1, 1, w.L), dtype=torch.float32, device="cuda:0")
    O = rr.rr_sparse_attn(Q, K, V, mask, lse=lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all()) and bool(torch.isfinite(lse).all())
    count = mask.row_count.cpu().numpy()[0, 0]
    _say(f"[full] 1M: density {count.sum() / (w.Nb * (w.Nb + 1) / 2):.4f}")
    rng = np.random.default_rng(5)
    rows = sorted({0, 1, 4095, 4096, 8190, 8191} | {int(v) for v in rng.integers(0, w.Nb, 6)})
    excused = 0
    for m in rows:
        ref, _, margin = oracle.estimate_row(x["Q"][0], x["K"][0], 0, m, w.S, w.B, tau, True)
        got = mask.dense[0, 0, m, : m + 1].cpu().numpy()
        diff = got != ref
        assert (margin[diff] < gu.MARGIN_TOL).all(), (m, int(diff.sum()))
        excused += int(diff.sum())
        assert not bool(mask.dense[0, 0, m, m + 1:].any())
        lst = mask.row_list[0, 0, m, : count[m]].cpu().numpy()
        assert np.array_equal(lst, np.nonzero(got)[0])
    _say(f"[full] 1M: {len(rows)} mask rows, {excused} excused blocks")
    mask_np_rows = {m: mask.dense[0, 0, m].cpu().numpy() for m in rows}
    worst = 0.0
    for m in rows:
        ref_O, ref_lse = oracle.attention_row_block(x["Q"][0], x["K"][0], x["V"][0], mask_np_rows[m], m, w.B)
        got = O[0, 0, m * w.B:(m + 1) * w.B].float().cpu().numpy().astype(np.float64)
        d = np.abs(got - ref_O)
        worst = max(worst, float(d.max()))
        assert d.max() <= gu.BF16_MAX_ABS and d.mean() <= gu.BF16_MEAN_ABS, m
        assert np.abs(lse[0, 0, m * w.B:(m + 1) * w.B].cpu().numpy() - ref_lse).max() < 2e-2
    _say(f"[full] 1M sparse: {len(rows)} query blocks, max abs {worst:.3e}")
    del mask
    Od = rr.rr_dense_attn(Q, K, V, w.B, lse=lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Od).all())
    full = np.ones(w.Nb, dtype=np.uint8)
    for m in (0, 8191):
        ref_O, _ = oracle.attention_row_block(x["Q"][0], x["K"][0], x["V"][0], full, m, w.B)
        d = np.abs(Od[0, 0, m * w.B:(m + 1) * w.B].float().cpu().numpy().astype(np.float64) - ref_O)
        assert d.max() <= gu.BF16_MAX_ABS and d.mean() <= gu.BF16_MEAN_ABS, m


def test_full_size_ragged_length():
    """cfg2 cut to 130 907 positions (1023 blocks: the last one holds 91 positions, 5 complete strides): masks
    of every head in full, sampled attention rows including the partial block of several heads."""
    import paper_2602_05853_amd as rr
    w = ri.get_config("cfg2")
    L = 128 * 1022 + 91
    Nb = 1023
    S, tau = 16, 0.9
    _say(f"[full] case=ragged L={L}")
    x = {k: np.ascontiguousarray(v[:, :L]) for k, v in ri.generate(w).items()}
    t = gu.to_device(x, w.dtype)
    Q, K, V = t["Q"], t["K"], t["V"]
    ws = torch.empty(rr.rr_workspace_bytes(Q, K, S, w.B), dtype=torch.uint8, device=Q.device)
    mask = rr.BlockMask.allocate(1, w.Hq, Nb, w.B, Q.device, dense=True, block_mass=True, Hkv=w.Hkv)
    rr.rr_estimate(Q, K, S, w.B, tau, out=mask, workspace=ws)
    torch.cuda.synchronize()
    del ws
    ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, S, w.B, tau, True)
    assert ref_mask.shape == (w.Hq, Nb, Nb)
    gu.check_mask_structures(mask)
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
    _say(f"[full] ragged: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5
    del ref_frac, ref_margin
    O = torch.full_like(Q, float("nan"))
    lse = torch.empty((1, w.Hq, L), dtype=torch.float32, device=Q.device)
    rr.rr_sparse_attn(Q, K, V, mask, O=O, lse=lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all()) and bool(torch.isfinite(lse).all())
    mask_np = mask.dense.cpu().numpy()[0]
    rng = np.random.default_rng(17)
    rows = {(0, Nb - 1), (w.Hq - 1, Nb - 1), (13, Nb - 1), (5, Nb - 2), (0, 0)}
    while len(rows) < 24:
        rows.add((int(rng.integers(w.Hq)), int(rng.integers(Nb))))
    # _check_rows slices whole blocks: the oracle returns 91 rows for the last one, so does the slice of O
    _check_rows(x, w, O, lse, mask_np, sorted(rows), "ragged sparse")
