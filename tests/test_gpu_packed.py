"""GPU parity of packed sequences (a batch of prompts of different lengths laid back to back, each a whole
number of blocks): estimation with a seq_first table, the sparse kernel on the block-diagonal mask, and
the packed dense baseline, against the oracle's sequence-by-sequence statement.  Same bar as the other
parity tests."""
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


def rr():
    import paper_2602_05853_amd as p
    return p


PACKED_CASES = {
    # name: (workload of the packed length, blocks per sequence, tau, protect, sink, recent, offset mode, layer)
    # MFMA score kernel: a workgroup's query blocks span several sequences; sequences start inside a 32-stride tile
    "mfma_R8": (ri.custom(L=128 * 18, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=201, logit_gain=2.5),
                [5, 1, 9, 3], 0.85, True, 0, 0, "head", 0),
    "mfma_R4_lane_blocks": (ri.custom(L=128 * 21, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=32, seed=202, logit_gain=2.5),
                            [3, 7, 1, 1, 9], 0.9, True, 1, 1, "hybrid", 3),
    "mfma_R32_no_protect": (ri.custom(L=128 * 9, Hq=4, Hkv=1, d=128, dtype="bf16", B=128, S=4, seed=203, logit_gain=2.5),
                            [2, 6, 1], 0.7, False, 0, 0, "head", 0),
    "mfma_R16_many_short": (ri.custom(L=128 * 24, Hq=6, Hkv=2, d=128, dtype="bf16", B=128, S=8, seed=204, logit_gain=3.0),
                            [1] * 7 + [10] + [1, 2, 4], 0.9, True, 0, 2, "head", 0),
    # long enough for the key split of the block-mass kernel (two launches, 5 chunks of key tiles per row group),
    # with sequence starts inside a chunk and chunks that lie wholly in front of a row's sequence
    "mfma_R32_key_split": (ri.custom(L=128 * 40, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=4, seed=208, logit_gain=2.5),
                           [14, 3, 23], 0.9, True, 0, 0, "head", 0),
    # generic kernels
    "generic_f32": (ri.custom(L=64 * 14, Hq=4, Hkv=2, d=64, dtype="f32", B=64, S=8, seed=205, logit_gain=2.5),
                    [2, 7, 1, 4], 0.6, False, 1, 0, "fixed", 0),
    "generic_bf16_many_blocks": (ri.custom(L=16 * 300, Hq=2, Hkv=1, d=64, dtype="bf16", B=16, S=8, seed=206, logit_gain=3.0),
                                        [120, 1, 179], 0.9, True, 0, 0, "head", 0),
    "one_sequence": (ri.custom(L=128 * 6, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=207, logit_gain=2.5),
                     [6], 0.9, True, 0, 0, "head", 0),
}


@pytest.mark.parametrize("name", list(PACKED_CASES))
def test_packed_estimate_and_attention_match_oracle(name):
    w, blocks, tau, protect, sink, recent, mode, layer = PACKED_CASES[name]
    assert sum(blocks) == w.Nb
    _say(f"[packed] case={name} L={w.L} Hq={w.Hq} Hkv={w.Hkv} d={w.d} {w.dtype} B={w.B} S={w.S} blocks={blocks}")
    x = ri.generate(w)
    ref_mask, ref_frac, ref_margin = oracle.estimate_packed(x["Q"], x["K"], w.S, w.B, tau, blocks, protect, mode, layer,
                                                            sink, recent)
    t = gu.to_device(x, w.dtype)
    p = rr()
    sf = p.packed_seq_first(blocks, "cuda:0")
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, tau, flags=1 if protect else 0, block_mass=True,
                         offset_mode=mode, layer=layer, sink_blocks=sink, recent_blocks=recent, seq_first=sf)
    torch.cuda.synchronize()
    dense = gu.check_mask_structures(mask)[0]
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
    _say(f"[packed] {name} estimate: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5
    # nothing outside a row's own sequence, whatever the margins say
    inside = oracle.packed_causal_block_mask(w.Hq, blocks).astype(bool)
    assert not dense[~inside].any()
    order = mask.row_order.cpu().numpy()[0]
    for kv in range(w.Hkv):
        assert np.array_equal(np.sort(order[kv]), np.arange(w.G * w.Nb))

    # sparse attention on the packed tensors with the mask as estimated on the device
    lse = torch.empty((1, w.Hq, w.L), dtype=torch.float32, device="cuda:0")
    O = p.rr_sparse_attn(t["Q"], t["K"], t["V"], mask, lse=lse)
    Od = p.rr_dense_attn_packed(t["Q"], t["K"], t["V"], w.B, sf)
    torch.cuda.synchronize()
    O_ref, lse_ref = oracle.sparse_attention(x["Q"], x["K"], x["V"], dense, w.B)
    Od_ref, _ = oracle.sparse_attention(x["Q"], x["K"], x["V"], inside.astype(np.uint8), w.B)
    for what, got, want in (("sparse", O, O_ref), ("dense", Od, Od_ref)):
        mx, mean = gu.attention_errors(got[0], want)
        _say(f"[packed] {name} {what}: max abs {mx:.3e} mean abs {mean:.3e}")
        if w.dtype == "bf16":
            assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS
        else:
            assert mx <= gu.F32_MAX_ABS
    assert np.abs(lse[0].cpu().numpy() - lse_ref).max() < (2e-2 if w.dtype == "bf16" else 1e-4)


def test_packed_attention_equals_the_sequences_run_one_by_one():
    """The rows of a packed call walk the same blocks in the same order as the rows of a call on the
    sequence alone, so the attention outputs are the same numbers."""
    w = ri.custom(L=128 * 12, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=211, logit_gain=2.5)
    blocks = [4, 1, 7]
    t = gu.to_device(ri.generate(w), w.dtype)
    p = rr()
    sf = p.packed_seq_first(blocks, "cuda:0")
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.8, seq_first=sf)
    O = p.rr_sparse_attn(t["Q"], t["K"], t["V"], mask)
    Od = p.rr_dense_attn_packed(t["Q"], t["K"], t["V"], w.B, sf)
    torch.cuda.synchronize()
    dense = mask.dense.cpu().numpy()[0]
    for (b0, b1) in oracle.sequence_block_ranges(blocks):
        sl = slice(b0 * w.B, b1 * w.B)
        q, k, v = (t[n][:, :, sl].contiguous() for n in "QKV")
        sub = gu.blockmask_from_dense(np.ascontiguousarray(dense[:, b0:b1, b0:b1]), w.B)
        O1 = p.rr_sparse_attn(q, k, v, sub)
        Od1 = p.rr_dense_attn(q, k, v, w.B)
        torch.cuda.synchronize()
        assert torch.equal(O1, O[:, :, sl]), (b0, b1)
        assert torch.equal(Od1, Od[:, :, sl]), (b0, b1)


def test_packed_ragged_lengths_do_not_depend_on_the_filler():
    """Sequences whose lengths are not multiples of B are filled up to a block boundary inside the packed
    tensors: masks are the same whatever the filler holds, and the outputs of real positions agree up to
    the rounding of P (a wave shares its lazy softmax reference among real and filler queries)."""
    B, S = 128, 16
    real = [600, 128, 1000, 77]
    blocks = [(n + B - 1) // B for n in real]
    w = ri.custom(L=B * sum(blocks), Hq=4, Hkv=2, d=128, dtype="bf16", B=B, S=S, seed=212, logit_gain=3.0)
    t = gu.to_device(ri.generate(w), w.dtype)
    p = rr()
    sf = p.packed_seq_first(blocks, "cuda:0")
    keep = torch.zeros(w.L, dtype=torch.bool, device="cuda:0")
    for (b0, _), n in zip(oracle.sequence_block_ranges(blocks), real):
        keep[b0 * B: b0 * B + n] = True
    outs = []
    for fill in (0.0, -2.5):
        q, k, v = (t[n].clone() for n in "QKV")
        for z in (q, k, v):
            z[:, :, ~keep, :] = fill
        mask = p.rr_estimate(q, k, S, B, 0.85, seq_first=sf)
        O = p.rr_sparse_attn(q, k, v, mask)
        torch.cuda.synchronize()
        outs.append((mask.dense.clone(), O[:, :, keep].clone()))
    assert torch.equal(outs[0][0], outs[1][0])
    diff = (outs[0][1].float() - outs[1][1].float()).abs()
    assert float(diff.max()) <= 1e-2 and float(diff.mean()) <= 1e-4


def test_packed_argument_errors_and_clamping():
    w = ri.custom(L=128 * 8, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=213)
    t = gu.to_device(ri.generate(w), w.dtype)
    p = rr()
    sf = p.packed_seq_first([3, 5], "cuda:0")
    # a query chunk and packed sequences do not combine
    qc = t["Q"][:, :, -256:].contiguous()
    with pytest.raises(p.RRError) as e:
        p.rr_estimate(qc, t["K"], w.S, w.B, 0.9, seq_first=sf)
    assert e.value.status == -4
    with pytest.raises(p.RRError) as e:
        p.rr_dense_attn_packed(qc, t["K"], t["V"], w.B, sf)
    assert e.value.status == -4
    with pytest.raises(p.RRError):
        p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9, seq_first=sf[:-1].contiguous())
    # a table with values outside [0, m] is clamped on the device: wrong rows, no fault
    bad = torch.tensor([0, 5, -3, 3, 9, 3, 100, 3], dtype=torch.int32, device="cuda:0")
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9, seq_first=bad)
    O = p.rr_dense_attn_packed(t["Q"], t["K"], t["V"], w.B, bad)
    torch.cuda.synchronize()
    gu.check_mask_structures(mask)
    assert bool(torch.isfinite(O.float()).all())
