"""Decode-stage extension / steps at arbitrary offsets: Q holds the last Lq positions of an L-token context,
Lq from one token to several blocks, starting anywhere.  The masks of the step are compared with the oracle's
reading of a step (rows estimated from the sampled positions the step holds; a row without any keeps every
causal block), the attention outputs with the rows q0 .. L-1 of the oracle's attention under the same mask,
the dense baseline with the library-pinned dense attention.  Positions in front of the step are poisoned in
the tensor the GPU reads from."""
import sys

import numpy as np
import pytest
import torch

import rr_inputs as ri
from oracle import rr_oracle as oracle
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _w(L, Hq, Hkv, d, dtype, B, S, seed):
    return ri.custom(L=L, Hq=Hq, Hkv=Hkv, d=d, dtype=dtype, B=B, S=S, tau=0.9, seed=seed, logit_gain=2.5)


# name: (workload, real length L, [q0 ...], tau, protect the last query block)
STEPS = {
    # MFMA kernels (bf16, d = 128, B = 128)
    "mfma_one_token_and_small_steps": (_w(1536, 8, 2, 128, "bf16", 128, 16, 31), 1536, [1535, 1534, 1529, 1520, 1472], 0.8, False),
    "mfma_steps_across_blocks": (_w(2048, 4, 2, 128, "bf16", 128, 16, 32), 2048, [1999, 1800, 1153, 640 + 77, 5], 0.9, False),
    "mfma_ragged_context": (_w(1536, 4, 4, 128, "bf16", 128, 8, 33), 1536 - 59, [1536 - 60, 1536 - 61, 1400, 1290, 1025], 0.85, False),
    # one and two new tokens (the decode kernel when the call has a workspace): two tokens in two different query
    # blocks; seven query heads per KV head (one token: 7 rows; two tokens: 14 rows, back on the matrix kernel)
    "mfma_decode_block_boundary": (_w(1536, 8, 2, 128, "bf16", 128, 16, 38), 1409, [1407, 1408], 0.8, False),
    "mfma_decode_seven_heads": (_w(1024, 7, 1, 128, "bf16", 128, 8, 39), 1019, [1018, 1017], 0.8, False),
    # a long context (256 key blocks: rows of several tiles, the row queue of the sparse launch in use)
    "mfma_32k_context": (_w(32768, 16, 4, 128, "bf16", 128, 16, 37), 32768, [32767, 32768 - 16, 32768 - 700], 0.9, False),
    # chunks of a long prompt (160 key blocks, several query blocks per head): with a workspace the long rows are
    # cut into parts of 64 list entries, short rows stay whole
    "mfma_chunks_of_a_long_prompt": (_w(20480, 4, 2, 128, "bf16", 128, 16, 46), 20480,
                                     [20480 - 300, 20480 - 1000, 20480 - 1024, 20480 - 2048 - 77], 0.9, False),
    "mfma_chunks_ragged_context": (_w(20480, 6, 2, 128, "bf16", 128, 8, 47), 20480 - 59, [20480 - 59 - 700, 20480 - 59 - 260], 0.9, False),
    "mfma_R4_protected": (_w(1024, 8, 1, 128, "bf16", 128, 32, 34), 1024, [1023, 1000, 900, 300], 0.9, True),
    # generic kernels
    "f32_d64_B64": (_w(1024, 4, 2, 64, "f32", 64, 8, 35), 1024, [1023, 1016, 1000, 777, 130, 3], 0.9, False),
    "bf16_d96_B32_ragged": (_w(512, 6, 3, 96, "bf16", 32, 4, 36), 512 - 13, [498, 490, 471, 300, 33], 0.8, False),
}


@pytest.mark.parametrize("name", list(STEPS))
def test_step_at_any_offset_matches_oracle(name):
    import paper_2602_05853_amd as p
    w, L, starts, tau, protect = STEPS[name]
    x = {k: np.ascontiguousarray(v[:, :L]) for k, v in ri.generate(w).items()}
    G, B, S = w.G, w.B, w.S
    Nb = -(-L // B)
    t = gu.to_device(x, w.dtype)
    tol_max, tol_mean = (gu.BF16_MAX_ABS, gu.BF16_MEAN_ABS) if w.dtype == "bf16" else (gu.F32_MAX_ABS, gu.F32_MAX_ABS)
    for q0 in starts:
        Lq = L - q0
        _say(f"[step] case={name} L={L} q0={q0} Lq={Lq} Hq={w.Hq} d={w.d} {w.dtype} B={B} S={S} tau={tau} protect={protect}")
        ref_mask, ref_frac, ref_margin = oracle.estimate_step(x["Q"], x["K"], q0, S, B, tau, protect)
        m0 = q0 // B
        rows = Nb - m0
        # the GPU reads the step's queries from a buffer of their own: nothing in front of q0 exists for it
        Qc = t["Q"][:, :, q0:, :].contiguous()
        mask = p.rr_estimate(Qc, t["K"], S, B, tau, flags=1 if protect else 0, block_mass=True)
        torch.cuda.synchronize()
        assert mask.dense.shape == (1, w.Hq, rows, Nb) and mask.row_count.shape == (1, w.Hq, rows)
        dense = mask.dense.cpu().numpy()[0]
        rep = oracle.compare_masks(ref_mask, ref_margin, ref_frac, dense, margin_tol=gu.MARGIN_TOL)
        rep["mass_max_abs_err"] = float(np.abs(mask.block_mass.cpu().numpy()[0] - ref_frac).max())
        rep["rows_without_estimate"] = int((~ref_frac.any(-1)).sum())
        _say(f"[step] {name} q0={q0}: {rep}")
        assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5
        count, lst = mask.row_count.cpu().numpy()[0], mask.row_list.cpu().numpy()[0]
        for h in range(w.Hq):
            for r in range(rows):
                assert np.array_equal(lst[h, r, :count[h, r]], np.nonzero(dense[h, r])[0])
        order = mask.row_order.cpu().numpy()[0]
        for kv in range(w.Hkv):
            assert np.array_equal(np.sort(order[kv]), np.arange(G * rows))

        lse = torch.full((1, w.Hq, Lq), float("nan"), dtype=torch.float32, device="cuda:0")
        O = torch.full_like(Qc, float("nan"))
        p.rr_sparse_attn(Qc, t["K"], t["V"], mask, O=O, lse=lse)
        Od = p.rr_dense_attn(Qc, t["K"], t["V"], B)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(O.float()).all()) and bool(torch.isfinite(lse).all())
        full_mask = oracle.causal_block_mask(w.Hq, Nb)
        full_mask[:, m0:] = dense
        need = [(h, m) for h in range(w.Hq) for m in range(m0, Nb)]
        ref = oracle.sparse_attention(x["Q"], x["K"], x["V"], full_mask, B, rows=need)
        refd = oracle.dense_attention(x["Q"], x["K"], x["V"], B, rows=need)
        O_ref = np.zeros((w.Hq, Lq, w.d))
        Od_ref = np.zeros((w.Hq, Lq, w.d))
        lse_ref = np.zeros((w.Hq, Lq))
        for (h, m) in need:
            lo, hi = max(m * B, q0), min((m + 1) * B, L)
            O_ref[h, lo - q0:hi - q0] = ref[(h, m)][0][lo - m * B:hi - m * B]
            lse_ref[h, lo - q0:hi - q0] = ref[(h, m)][1][lo - m * B:hi - m * B]
            Od_ref[h, lo - q0:hi - q0] = refd[(h, m)][0][lo - m * B:hi - m * B]
        checks = [("sparse", O, O_ref), ("dense", Od, Od_ref)]
        # the entry points with a workspace: where the call is split (few rows, long lists) the shares of a row's
        # block list are computed by several workgroups and merged; the same bar against the oracle applies
        need_ws = p.rr_attn_workspace_bytes(Qc, t["K"], B)
        if need_ws:
            wsa = torch.empty(need_ws, dtype=torch.uint8, device="cuda:0")
            lse2 = torch.full_like(lse, float("nan"))
            O2 = torch.full_like(Qc, float("nan"))
            p.rr_sparse_attn(Qc, t["K"], t["V"], mask, O=O2, lse=lse2, workspace=wsa)
            Od2 = torch.full_like(Qc, float("nan"))
            p.rr_dense_attn(Qc, t["K"], t["V"], B, O=Od2, workspace=wsa)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(O2.float()).all()) and bool(torch.isfinite(lse2).all())
            checks += [("sparse, split", O2, O_ref), ("dense, split", Od2, Od_ref)]
            assert np.abs(lse2[0].cpu().numpy() - lse_ref).max() < 2e-2
            _say(f"[step] {name} q0={q0}: split workspace {need_ws} bytes, split vs one workgroup per row max abs "
                 f"{float((O2.float() - O.float()).abs().max()):.3e}")
        for label, got, want in checks:
            mx, mean = gu.attention_errors(got[0], want)
            _say(f"[step] {name} q0={q0} {label}: max abs {mx:.3e} mean abs {mean:.3e}")
            assert mx <= tol_max and mean <= tol_mean
        assert np.abs(lse[0].cpu().numpy() - lse_ref).max() < (2e-2 if w.dtype == "bf16" else 1e-4)


def test_one_token_steps_are_dense_unless_the_token_is_a_sampled_position():
    """The reading of a one-token step, head by head: the new token (the last position of a stride here) is the
    sampled position of that stride only for heads with h mod S = 0; every other head has no sampled query and
    must list every causal block, which is how the paper decodes."""
    import paper_2602_05853_amd as p
    w = _w(1024, 8, 2, 128, "bf16", 128, 4, 41)
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    Qc = t["Q"][:, :, 1023:, :].contiguous()
    mask = p.rr_estimate(Qc, t["K"], w.S, w.B, 0.5, flags=0)
    torch.cuda.synchronize()
    count = mask.row_count.cpu().numpy()[0, :, 0]
    _say(f"[step] one token: selected blocks per head {count.tolist()}")
    for h in range(w.Hq):
        if h % w.S == 0:
            assert 1 <= count[h] < 8
        else:
            assert count[h] == 8


def test_workspace_attention_is_the_plain_call_where_nothing_is_split_and_checks_its_workspace():
    import paper_2602_05853_amd as p
    from paper_2602_05853_amd import binding as bd
    w = _w(4096, 8, 2, 128, "bf16", 128, 16, 43)
    t = gu.to_device(ri.generate(w), w.dtype)
    # a whole prefill: 256 rows, nothing to split
    assert p.rr_attn_workspace_bytes(t["Q"], t["K"], w.B) == 0
    # a step of 100 tokens: 8 rows with lists of up to 32 blocks
    Qc = t["Q"][:, :, 4096 - 100:].contiguous()
    need = p.rr_attn_workspace_bytes(Qc, t["K"], w.B)
    assert need > 0 and need % 256 == 0
    mask = p.rr_estimate(Qc, t["K"], w.S, w.B, 0.9, flags=0)
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(bd.RRError) as err:
        p.rr_sparse_attn(Qc, t["K"], t["V"], mask, workspace=small)
    assert err.value.status == bd.RR_ERR_WORKSPACE
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    O1 = p.rr_sparse_attn(Qc, t["K"], t["V"], mask)
    O2 = p.rr_sparse_attn(Qc, t["K"], t["V"], mask, workspace=ws)
    torch.cuda.synchronize()
    assert float((O1.float() - O2.float()).abs().max()) < 2e-2
    # two sequences in the batch, 3 query heads per KV head, a step that starts inside a block and a context that
    # ends inside one: every part of every row lands in its own place of the workspace
    wb = _w(4096, 6, 2, 128, "bf16", 128, 16, 45)
    xb = ri.generate(wb)
    Lb = 4096 - 21
    tb = {k: torch.from_numpy(np.stack([v[:, :Lb], v[:, :Lb][:, ::-1].copy()])).to(torch.bfloat16).to("cuda:0")
          for k, v in xb.items()}
    Qb = tb["Q"][:, :, Lb - 200:].contiguous()
    needb = p.rr_attn_workspace_bytes(Qb, tb["K"], wb.B)
    assert needb > 0
    maskb = p.rr_estimate(Qb, tb["K"], wb.S, wb.B, 0.9, flags=0)
    wsb = torch.empty(needb, dtype=torch.uint8, device="cuda:0")
    for f in (lambda **kw: p.rr_sparse_attn(Qb, tb["K"], tb["V"], maskb, **kw),
              lambda **kw: p.rr_dense_attn(Qb, tb["K"], tb["V"], wb.B, **kw)):
        l1 = torch.empty((2, wb.Hq, 200), dtype=torch.float32, device="cuda:0")
        l2 = torch.empty_like(l1)
        A = f(lse=l1)
        Bs = f(lse=l2, workspace=wsb)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(Bs.float()).all())
        assert float((A.float() - Bs.float()).abs().max()) < 2e-2 and float((l1 - l2).abs().max()) < 1e-3
    # one and two new tokens for both sequences of the batch: the decode kernel
    for T in (1, 2):
        Qd = tb["Q"][:, :, Lb - T:].contiguous()
        maskd = p.rr_estimate(Qd, tb["K"], wb.S, wb.B, 0.9, flags=0)
        wsd = torch.empty(p.rr_attn_workspace_bytes(Qd, tb["K"], wb.B), dtype=torch.uint8, device="cuda:0")
        for f in (lambda **kw: p.rr_sparse_attn(Qd, tb["K"], tb["V"], maskd, **kw),
                  lambda **kw: p.rr_dense_attn(Qd, tb["K"], tb["V"], wb.B, **kw)):
            l1 = torch.empty((2, wb.Hq, T), dtype=torch.float32, device="cuda:0")
            l2 = torch.full_like(l1, float("nan"))
            A = f(lse=l1)
            Bs = f(lse=l2, workspace=wsd)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(Bs.float()).all())
            assert float((A.float() - Bs.float()).abs().max()) < 2e-2 and float((l1 - l2).abs().max()) < 1e-2
    # fp32 tensors go to the generic kernel: no split, a workspace is ignored
    w32 = _w(1024, 4, 2, 64, "f32", 64, 8, 44)
    t32 = gu.to_device(ri.generate(w32), w32.dtype)
    Q32 = t32["Q"][:, :, 1000:].contiguous()
    assert p.rr_attn_workspace_bytes(Q32, t32["K"], w32.B) == 0
    a = p.rr_dense_attn(Q32, t32["K"], t32["V"], w32.B)
    b_ = p.rr_dense_attn(Q32, t32["K"], t32["V"], w32.B, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b_)


def test_chunk_of_a_long_prompt_when_the_slots_run_out():
    """A chunk of 8192 tokens at a 64K context, dense: 256 rows of 449-512 blocks, eight parts each, against 1024
    slots -- the plan cuts the longest rows and leaves the others whole.  Every row against the call without a
    workspace, a sample of rows against the oracle; two sequences in the batch."""
    import paper_2602_05853_amd as p
    w = _w(65536, 4, 2, 128, "bf16", 128, 16, 48)
    x = ri.generate(w)
    L, B, Lq = w.L, w.B, 8192
    t = {k: torch.from_numpy(np.stack([v, v[:, ::-1].copy()])).to(torch.bfloat16).to("cuda:0") for k, v in x.items()}
    Qc = t["Q"][:, :, L - Lq:].contiguous()
    need = p.rr_attn_workspace_bytes(Qc, t["K"], B)
    rows, slots = 2 * w.Hq * (Lq // B), 2048
    assert need == 256 + rows * 4 + slots * 4 + slots // 2 * 4 + slots * 128 * 4 + slots * 128 * 128 * 4
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    l1 = torch.empty((2, w.Hq, Lq), dtype=torch.float32, device="cuda:0")
    l2 = torch.full_like(l1, float("nan"))
    _say(f"[chunk] dense chunk of {Lq} tokens at L={L}: {rows} rows, {slots} slots")
    A = p.rr_dense_attn(Qc, t["K"], t["V"], B, lse=l1)
    Bs = torch.full_like(Qc, float("nan"))
    p.rr_dense_attn(Qc, t["K"], t["V"], B, O=Bs, lse=l2, workspace=ws)
    torch.cuda.synchronize()
    used = int(ws[:4].cpu().view(torch.int32)[0])
    _say(f"[chunk] slots in use {used}")
    assert slots - 8 < used <= slots                        # the slots ran out: some rows of eight parts stayed whole
    assert bool(torch.isfinite(Bs.float()).all()) and bool(torch.isfinite(l2).all())
    assert float((A.float() - Bs.float()).abs().max()) < 2e-2 and float((l1 - l2).abs().max()) < 1e-3
    Nb, m0 = L // B, (L - Lq) // B
    rng = np.random.default_rng(5)
    need_rows = sorted({(0, Nb - 1), (w.Hq - 1, m0)} | {(int(rng.integers(w.Hq)), int(rng.integers(m0, Nb))) for _ in range(10)})
    ref = oracle.dense_attention(x["Q"], x["K"], x["V"], B, rows=need_rows)
    for (h, m) in need_rows:
        got = Bs[0, h, (m - m0) * B:(m - m0 + 1) * B]
        mx, mean = gu.attention_errors(got, ref[(h, m)][0])
        assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS, (h, m)
    # the sparse call on the same chunk (lists of very different lengths)
    mask = p.rr_estimate(Qc, t["K"], w.S, B, 0.9, flags=0)
    O1 = p.rr_sparse_attn(Qc, t["K"], t["V"], mask, lse=l1)
    O2 = torch.full_like(Qc, float("nan"))
    p.rr_sparse_attn(Qc, t["K"], t["V"], mask, O=O2, lse=l2, workspace=ws)
    torch.cuda.synchronize()
    _say(f"[chunk] sparse: slots in use {int(ws[:4].cpu().view(torch.int32)[0])}, longest row {int(mask.row_count.max())}")
    assert float((O1.float() - O2.float()).abs().max()) < 2e-2 and float((l1 - l2).abs().max()) < 1e-3


def test_stride_sums_kept_from_call_to_call_give_the_same_masks():
    """A context that grows call by call (chunks of a prompt, then single tokens), the stride key sums kept in the
    workspace (ksum_capacity / ksum_valid): every call must give, bit for bit, what the same call gives when it forms
    all sums itself -- at aligned lengths, at lengths that end inside a stride and inside a block, after a call
    that added nothing to a stride, and again from scratch (ksum_valid = 0) in a used workspace."""
    import paper_2602_05853_amd as p
    w = _w(8192, 8, 2, 128, "bf16", 128, 16, 49)
    t = gu.to_device(ri.generate(w), w.dtype)
    cap, S, B = 8192, w.S, w.B
    lengths = [1024, 2048 + 77, 2048 + 77 + 300, 2048 + 77 + 301, 5000, 5001, 5002, 8192 - 59, 8192]
    longest = max(b - a for a, b in zip([0] + lengths[:-1], lengths))
    ws = torch.empty(p.rr_workspace_bytes(t["Q"][:, :, :longest].contiguous(), t["K"], S, B), dtype=torch.uint8, device="cuda:0")
    ws.fill_(0xFF)
    prev = 0
    for i, L in enumerate(lengths + [3000]):
        if L < prev:
            prev = 0                                         # a new prompt in the same workspace: nothing is valid
        Kv = t["K"][:, :, :L]
        Qc = t["Q"][:, :, prev:L].contiguous()
        kept = p.rr_estimate(Qc, Kv, S, B, 0.9, flags=0, workspace=ws, block_mass=True, ksum_capacity=cap, ksum_valid=prev)
        plain = p.rr_estimate(Qc, Kv, S, B, 0.9, flags=0, block_mass=True)
        torch.cuda.synchronize()
        _say(f"[kept sums] call {i}: L={L} new positions {L - prev}, selected {int(plain.row_count.sum())}")
        assert torch.equal(kept.row_count, plain.row_count) and torch.equal(kept.dense, plain.dense)
        assert torch.equal(kept.block_mass, plain.block_mass)
        cnt = plain.row_count.flatten().tolist()
        kl, pl = kept.row_list.reshape(len(cnt), -1), plain.row_list.reshape(len(cnt), -1)
        for r, c in enumerate(cnt):
            assert torch.equal(kl[r, :c], pl[r, :c])
        prev = L
    # a workspace sized for the call alone is too small for the capacity layout
    small = torch.empty(p.rr_workspace_bytes(Qc, Kv, S, B), dtype=torch.uint8, device="cuda:0")
    from paper_2602_05853_amd import binding as bd
    with pytest.raises(bd.RRError) as err:
        p.rr_estimate(Qc, Kv, S, B, 0.9, flags=0, workspace=small, ksum_capacity=cap, ksum_valid=0)
    assert err.value.status == bd.RR_ERR_WORKSPACE


def test_random_steps_and_chunks_with_a_workspace_agree_with_the_plain_calls():
    """Consistency, not parity (the plain calls are what the other tests hold against the oracle): 40 seeded random
    geometries -- one and two tokens, short steps, chunks; 1-8 query heads per KV head, batches, contexts that end
    inside a block -- through the entry points with a workspace (decode kernel, equal shares, planned launches)
    against the same calls without one."""
    import random
    import paper_2602_05853_amd as p
    rnd = random.Random(2602)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(5853)
    taken = {}
    for case in range(40):
        Hkv, G = rnd.choice([1, 2, 3, 4]), rnd.choice([1, 2, 3, 4, 5, 7, 8])
        Hq, batch = Hkv * G, rnd.choice([1, 1, 2])
        L = rnd.choice([300, 1500, 4096, 9000, 16384, 20000]) - rnd.choice([0, 0, 1, 59, 127])
        kind = rnd.choice(["one token", "two tokens", "step", "chunk", "chunk"])
        Lq = {"one token": 1, "two tokens": 2, "step": rnd.choice([3, 17, 100, 128]),
              "chunk": rnd.choice([129, 300, 1000, 2048])}[kind]
        S, tau = rnd.choice([4, 8, 16, 32]), rnd.choice([0.5, 0.8, 0.9, 0.95])
        if Lq >= L or G * (128 // S) > 256:
            continue
        _say(f"[ws] case {case}: {kind} batch={batch} Hq={Hq} Hkv={Hkv} L={L} Lq={Lq} S={S} tau={tau}")
        Q = (torch.randn(batch, Hq, L, 128, device="cuda:0", generator=gen) * 1.5).to(torch.bfloat16)
        K = (torch.randn(batch, Hkv, L, 128, device="cuda:0", generator=gen) * 1.5).to(torch.bfloat16)
        V = torch.randn(batch, Hkv, L, 128, device="cuda:0", generator=gen).to(torch.bfloat16)
        Qc = Q[:, :, L - Lq:].contiguous()
        mask = p.rr_estimate(Qc, K, S, 128, tau, flags=0)
        need = p.rr_attn_workspace_bytes(Qc, K, 128)
        taken[(kind, need > 0)] = taken.get((kind, need > 0), 0) + 1
        if not need:
            continue
        ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        ws.fill_(0xFF)
        for f in (lambda **kw: p.rr_sparse_attn(Qc, K, V, mask, **kw), lambda **kw: p.rr_dense_attn(Qc, K, V, 128, **kw)):
            l1 = torch.full((batch, Hq, Lq), float("nan"), device="cuda:0")
            l2 = torch.full_like(l1, float("nan"))
            A = f(lse=l1)
            Bv = torch.full_like(Qc, float("nan"))
            f(O=Bv, lse=l2, workspace=ws)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(Bv.float()).all()) and bool(torch.isfinite(l2).all()), case
            assert float((A.float() - Bv.float()).abs().max()) < 2e-2 and float((l1 - l2).abs().max()) < 1e-2, case
    _say(f"[ws] forms taken: {taken}")
    assert sum(v for (k, used), v in taken.items() if used) >= 20
