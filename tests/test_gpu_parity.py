"""GPU parity: the HIP library, called through its C ABI, against the fp64 CPU oracle on the same
seeded inputs, element by element.  Sizes are chosen so the oracle finishes in seconds while a
row still spans several tiles (several key chunks, several key blocks, more than one wave's rows).

Bar: block masks bit-exact except blocks whose cumulative-mass margin to tau is below 1e-4
(counted and printed); attention outputs within max abs 2e-2 / mean abs 2e-3 for bf16 tensors and
max abs 1e-4 for fp32 tensors (the generic kernels are fp32 throughout).
"""
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


EST_CASES = {
    # name: (workload, tau, protect)
    "cfg0_f32": (ri.get_config("cfg0"), 0.9, True),
    "bf16_R8": (ri.custom(L=2048, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=11, logit_gain=2.5), 0.9, True),
    "bf16_R16_tau95": (ri.custom(L=1024, Hq=4, Hkv=4, d=64, dtype="bf16", B=64, S=4, seed=12, logit_gain=2.5), 0.95, True),
    "f32_S1_R32": (ri.custom(L=256, Hq=3, Hkv=1, d=40, dtype="f32", B=32, S=1, seed=13), 0.8, True),
    "f32_S_eq_B": (ri.custom(L=512, Hq=2, Hkv=2, d=64, dtype="f32", B=16, S=16, seed=14), 0.7, True),
    "bf16_R3_odd": (ri.custom(L=768, Hq=6, Hkv=3, d=64, dtype="bf16", B=48, S=16, seed=15, logit_gain=2.0), 0.9, True),
    "tau_one": (ri.custom(L=512, Hq=2, Hkv=1, d=64, dtype="bf16", B=64, S=8, seed=16), 1.0, True),
    # S = 1: every query sampled, every key its own stride -- the exact block mass of full attention (R = B = 128)
    "exact_mass_S1_B128_bf16": (ri.custom(L=1024, Hq=2, Hkv=1, d=128, dtype="bf16", B=128, S=1, seed=21, logit_gain=2.5), 0.9, True),
    "exact_mass_S1_B128_f32": (ri.custom(L=640, Hq=2, Hkv=2, d=64, dtype="f32", B=128, S=1, seed=22, logit_gain=2.0), 0.8, False),
    "no_protect": (ri.custom(L=1024, Hq=4, Hkv=2, d=64, dtype="f32", B=64, S=8, seed=17, logit_gain=2.5), 0.6, False),
    "single_block": (ri.custom(L=128, Hq=2, Hkv=1, d=64, dtype="bf16", B=128, S=16, seed=18), 0.9, True),
    "many_blocks": (ri.custom(L=8192, Hq=2, Hkv=1, d=64, dtype="bf16", B=16, S=8, seed=19, logit_gain=3.0), 0.9, True),
    # bf16, d = 128, R in {4, 8, 16, 32}: the MFMA stride-score kernel.  Lane-local blocks (R = 4), groups
    # whose rows do not fill the 256-row workgroup (G*R = 48), a full workgroup per query block (G*R = 256),
    # a stride count that is not a multiple of the 32-stride tile, a ragged last group of query blocks,
    # and G*R = 512 which falls back to the generic kernel.
    "mfma_R4_S32": (ri.custom(L=4096, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=32, seed=41, logit_gain=2.5), 0.9, True),
    "mfma_R4_B64": (ri.custom(L=1024, Hq=8, Hkv=8, d=128, dtype="bf16", B=64, S=16, seed=42, logit_gain=2.5), 0.85, True),
    "mfma_R16_G3": (ri.custom(L=2048, Hq=6, Hkv=2, d=128, dtype="bf16", B=128, S=8, seed=43, logit_gain=2.5), 0.9, True),
    "mfma_R32_G8": (ri.custom(L=1536, Hq=8, Hkv=1, d=128, dtype="bf16", B=128, S=4, seed=44, logit_gain=2.5), 0.9, True),
    "mfma_R8_ragged": (ri.custom(L=640, Hq=2, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=45, logit_gain=2.0), 0.9, False),
    "mfma_R8_groups": (ri.custom(L=128 * 37, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=46, logit_gain=3.0), 0.95, True),
    "generic_G16_R32": (ri.custom(L=512, Hq=16, Hkv=1, d=128, dtype="bf16", B=128, S=4, seed=47, logit_gain=2.0), 0.9, True),
}


@pytest.mark.parametrize("name", list(EST_CASES))
def test_estimate_matches_oracle(name):
    w, tau, protect = EST_CASES[name]
    _say(f"[estimate] case={name} L={w.L} Hq={w.Hq} Hkv={w.Hkv} d={w.d} {w.dtype} B={w.B} S={w.S} tau={tau}")
    x = ri.generate(w)
    ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, w.S, w.B, tau, protect)
    t = gu.to_device(x, w.dtype)
    mask = rr().rr_estimate(t["Q"], t["K"], w.S, w.B, tau, flags=1 if protect else 0, block_mass=True)
    torch.cuda.synchronize()
    gu.check_mask_structures(mask)
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
    _say(f"[estimate] {name}: {rep}")
    assert rep["failed"] == 0
    assert rep["mass_max_abs_err"] < 2e-5
    if tau >= 1.0:
        assert rep["mismatch"] == 0


VARIANT_CASES = {
    # name: (workload, tau, offset mode, layer, sink blocks, recent blocks)
    "mfma_fixed": (ri.custom(L=2048, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=61, logit_gain=2.5), 0.9, "fixed", 0, 0, 0),
    "mfma_layer5": (ri.custom(L=2048, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=62, logit_gain=2.5), 0.9, "layer", 5, 0, 0),
    "mfma_hybrid19_sink_recent": (ri.custom(L=4096, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=8, seed=63, logit_gain=3.0), 0.8, "hybrid", 19, 1, 2),
    "generic_hybrid3": (ri.custom(L=1024, Hq=4, Hkv=2, d=64, dtype="f32", B=64, S=8, seed=64, logit_gain=2.5), 0.9, "hybrid", 3, 0, 0),
    "generic_layer_sink_recent": (ri.custom(L=1024, Hq=6, Hkv=3, d=64, dtype="bf16", B=64, S=16, seed=65, logit_gain=2.5), 0.7, "layer", 7, 2, 1),
    "head_with_recent_only": (ri.custom(L=1536, Hq=4, Hkv=4, d=128, dtype="bf16", B=128, S=32, seed=66, logit_gain=2.5), 0.6, "head", 0, 0, 3),
}


@pytest.mark.parametrize("name", list(VARIANT_CASES))
def test_estimate_variants_match_oracle(name):
    """Offset schedules and sink / recent protection of the ablations (Sec. 4) through rr_estimate_ex."""
    w, tau, mode, layer, sink, recent = VARIANT_CASES[name]
    _say(f"[variant] case={name} L={w.L} Hq={w.Hq} d={w.d} {w.dtype} B={w.B} S={w.S} tau={tau} {mode} layer={layer} "
         f"sink={sink} recent={recent}")
    x = ri.generate(w)
    G = w.G
    outs = [oracle.estimate_head(x["Q"][h], x["K"][h // G], h, w.S, w.B, tau, True, mode, layer, sink, recent)
            for h in range(w.Hq)]
    ref_mask, ref_frac, ref_margin = (np.stack([o[i] for o in outs]) for i in range(3))
    t = gu.to_device(x, w.dtype)
    mask = rr().rr_estimate(t["Q"], t["K"], w.S, w.B, tau, block_mass=True, offset_mode=mode, layer=layer,
                            sink_blocks=sink, recent_blocks=recent)
    torch.cuda.synchronize()
    gu.check_mask_structures(mask)
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
    _say(f"[variant] {name}: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5
    if mode != "head":
        # the variant must actually differ from the head rule on these inputs
        base = rr().rr_estimate(t["Q"], t["K"], w.S, w.B, tau, sink_blocks=sink, recent_blocks=recent)
        torch.cuda.synchronize()
        assert not torch.equal(base.dense, mask.dense)


DIAG_CASES = {
    # name: (workload, tau, offset mode, layer, blocks per packed sequence or None)
    "mfma_R8": (ri.custom(L=2048, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=71, logit_gain=2.5), 0.9, "head", 0, None),
    "mfma_R4_hybrid": (ri.custom(L=128 * 11, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=32, seed=72, logit_gain=2.5), 0.85, "hybrid", 7, None),
    "mfma_R32_packed": (ri.custom(L=128 * 9, Hq=4, Hkv=1, d=128, dtype="bf16", B=128, S=4, seed=73, logit_gain=2.5), 0.8, "head", 0, [2, 6, 1]),
    # (the same with the key tiles of a row group split over several workgroups: two launches of the block-mass kernel)
    "mfma_R32_packed_key_split": (ri.custom(L=128 * 40, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=4, seed=76, logit_gain=2.5), 0.85, "head", 0, [9, 31]),
    "generic_f32": (ri.custom(L=1024, Hq=6, Hkv=2, d=64, dtype="f32", B=64, S=8, seed=74, logit_gain=2.5), 0.7, "head", 0, None),
    "generic_bf16_S_eq_B": (ri.custom(L=512, Hq=4, Hkv=4, d=64, dtype="bf16", B=16, S=16, seed=75, logit_gain=2.0), 0.8, "layer", 3, [8, 24]),
}


@pytest.mark.parametrize("name", list(DIAG_CASES))
def test_estimate_token_exact_diagonal_matches_oracle(name):
    """RR_FLAG_DIAGONAL_TOKEN: the sampled query's own stride is summed up to the query's position only."""
    w, tau, mode, layer, blocks = DIAG_CASES[name]
    _say(f"[diag] case={name} L={w.L} Hq={w.Hq} d={w.d} {w.dtype} B={w.B} S={w.S} tau={tau} {mode} packed={blocks}")
    x = ri.generate(w)
    p = rr()
    ref_mask, ref_frac, ref_margin = oracle.estimate_packed(x["Q"], x["K"], w.S, w.B, tau, blocks or [w.Nb], True, mode, layer,
                                                            0, 0, "token")
    t = gu.to_device(x, w.dtype)
    sf = p.packed_seq_first(blocks, "cuda:0") if blocks else None
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, tau, flags=p.RR_FLAG_PROTECT_LAST | p.RR_FLAG_DIAGONAL_TOKEN,
                         block_mass=True, offset_mode=mode, layer=layer, seq_first=sf)
    torch.cuda.synchronize()
    gu.check_mask_structures(mask)
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
    _say(f"[diag] {name}: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5
    # the rule must matter on these inputs: the block mass differs from the whole-stride reading
    base = p.rr_estimate(t["Q"], t["K"], w.S, w.B, tau, block_mass=True, offset_mode=mode, layer=layer, seq_first=sf)
    torch.cuda.synchronize()
    assert float((base.block_mass - mask.block_mass).abs().max()) > 1e-4


def test_estimate_state_in_workspace_and_layout():
    """A row whose softmax state exceeds LDS goes through the workspace; tensors stored [b, L, H, d]."""
    w = ri.custom(L=65536, Hq=1, Hkv=1, d=64, dtype="bf16", B=64, S=4, seed=21, logit_gain=3.0)
    _say(f"[estimate] case=workspace_state L={w.L} B={w.B} S={w.S}")
    x = ri.generate(w)
    ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, w.S, w.B, 0.9, True, threads=1)
    t = gu.to_device(x, w.dtype, layout="blhd")
    p = rr()
    assert p.rr_workspace_bytes(t["Q"], t["K"], w.S, w.B) > w.Hkv * w.Ls * w.d * 4 + 1024
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9, block_mass=True)
    torch.cuda.synchronize()
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, 0.9)
    _say(f"[estimate] workspace_state: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5


def test_estimate_batch_two():
    """Batch is an independent outer dimension."""
    ws = [ri.custom(L=1024, Hq=4, Hkv=2, d=64, dtype="bf16", B=64, S=8, seed=s, logit_gain=2.5) for s in (31, 32)]
    xs = [ri.generate(w) for w in ws]
    dev = [gu.to_device(x, "bf16") for x in xs]
    Q = torch.cat([d["Q"] for d in dev], 0)
    K = torch.cat([d["K"] for d in dev], 0)
    mask = rr().rr_estimate(Q, K, 8, 64, 0.9, block_mass=True)
    torch.cuda.synchronize()
    dense = gu.check_mask_structures(mask)
    for b, x in enumerate(xs):
        ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, 8, 64, 0.9)
        rep = oracle.compare_masks(ref_mask, ref_margin, ref_frac, dense[b], margin_tol=gu.MARGIN_TOL)
        _say(f"[estimate] batch element {b}: {rep}")
        assert rep["failed"] == 0


def test_estimate_mfma_batch_two_strided():
    """MFMA score kernel with batch 2 and tensors stored [b, L, H, d] (head stride below row stride)."""
    ws = [ri.custom(L=1536, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=s, logit_gain=2.5) for s in (33, 34)]
    xs = [ri.generate(w) for w in ws]
    dev = [gu.to_device(x, "bf16", layout="blhd") for x in xs]
    Q = torch.cat([d["Q"].permute(0, 2, 1, 3) for d in dev], 0).contiguous().permute(0, 2, 1, 3)
    K = torch.cat([d["K"].permute(0, 2, 1, 3) for d in dev], 0).contiguous().permute(0, 2, 1, 3)
    assert Q.stride(1) == 128 and Q.shape == (2, 4, 1536, 128)
    mask = rr().rr_estimate(Q, K, 16, 128, 0.9, block_mass=True)
    torch.cuda.synchronize()
    dense = gu.check_mask_structures(mask)
    for b, x in enumerate(xs):
        ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, 16, 128, 0.9)
        rep = oracle.compare_masks(ref_mask, ref_margin, ref_frac, dense[b], margin_tol=gu.MARGIN_TOL)
        _say(f"[estimate] mfma batch element {b}: {rep}")
        assert rep["failed"] == 0
        assert np.abs(mask.block_mass.cpu().numpy()[b] - ref_frac).max() < 2e-5


def test_estimate_is_deterministic():
    w = EST_CASES["bf16_R8"][0]
    t = gu.to_device(ri.generate(w), w.dtype)
    a = rr().rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9, block_mass=True)
    b = rr().rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9, block_mass=True)
    torch.cuda.synchronize()
    assert torch.equal(a.dense, b.dense) and torch.equal(a.block_mass, b.block_mass)
    assert torch.equal(a.row_count, b.row_count)


# ------------------------------------------------------------------------------------------------

def _random_mask(H, Nb, seed, p=0.5):
    rng = np.random.default_rng(seed)
    m = (rng.random((H, Nb, Nb)) < p).astype(np.uint8)
    m[:, np.arange(Nb), np.arange(Nb)] = 1
    m *= np.tril(np.ones((Nb, Nb), dtype=np.uint8))
    if Nb > 3:
        m[0, 2, 2] = 0          # a row without its diagonal block
        m[0, 2, 0] = 1
        m[H - 1, 3, :] = 0      # a row with nothing selected: O = 0, lse = -inf
    return m


ATTN_CASES = {
    # name: (workload, kernel family, mask kind)
    "generic_f32_cfg0": (ri.get_config("cfg0"), "estimate"),
    "generic_bf16_B64_d128": (ri.custom(L=512, Hq=4, Hkv=2, d=128, dtype="bf16", B=64, S=8, seed=41, logit_gain=2.0), "random"),
    "generic_f32_B32_d40": (ri.custom(L=256, Hq=3, Hkv=1, d=40, dtype="f32", B=32, S=4, seed=42), "random"),
    "mfma_groups2": (ri.custom(L=2048, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=43, logit_gain=2.5), "estimate"),
    "mfma_groups8": (ri.custom(L=1024, Hq=16, Hkv=8, d=128, dtype="bf16", B=128, S=16, seed=44, logit_gain=2.5), "random"),
    "mfma_groups3": (ri.custom(L=1536, Hq=6, Hkv=3, d=128, dtype="bf16", B=128, S=16, seed=45, logit_gain=2.0), "random"),
    "mfma_single_block": (ri.custom(L=128, Hq=2, Hkv=1, d=128, dtype="bf16", B=128, S=16, seed=46), "random"),
}


@pytest.mark.parametrize("name", list(ATTN_CASES))
def test_sparse_and_dense_attention_match_oracle(name):
    w, kind = ATTN_CASES[name]
    _say(f"[attn] case={name} L={w.L} Hq={w.Hq} Hkv={w.Hkv} d={w.d} {w.dtype} B={w.B} mask={kind}")
    x = ri.generate(w)
    if kind == "estimate":
        mask_np = gu.oracle_estimate(x, w.S, w.B, w.tau)[0]
    else:
        mask_np = _random_mask(w.Hq, w.Nb, seed=w.seed)
    t = gu.to_device(x, w.dtype)
    p = rr()
    bm = gu.blockmask_from_dense(mask_np, w.B)
    lse = torch.empty((1, w.Hq, w.L), dtype=torch.float32, device="cuda:0")
    O = p.rr_sparse_attn(t["Q"], t["K"], t["V"], bm, lse=lse)
    torch.cuda.synchronize()
    O_ref, lse_ref = oracle.sparse_attention(x["Q"], x["K"], x["V"], mask_np, w.B)
    mx, mean = gu.attention_errors(O[0], O_ref)
    _say(f"[attn] {name} sparse: max abs {mx:.3e} mean abs {mean:.3e}")
    if w.dtype == "bf16":
        assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS
    else:
        assert mx <= gu.F32_MAX_ABS
    lse_gpu = lse[0].cpu().numpy().astype(np.float64)
    empty = np.isneginf(lse_ref)
    assert np.array_equal(np.isneginf(lse_gpu), empty)
    assert np.abs(lse_gpu[~empty] - lse_ref[~empty]).max() < (2e-2 if w.dtype == "bf16" else 1e-4)
    assert (O[0].float().cpu().numpy()[empty] == 0).all()

    Od = p.rr_dense_attn(t["Q"], t["K"], t["V"], w.B)
    torch.cuda.synchronize()
    Od_ref, _ = oracle.dense_attention(x["Q"], x["K"], x["V"], w.B)
    mx, mean = gu.attention_errors(Od[0], Od_ref)
    _say(f"[attn] {name} dense: max abs {mx:.3e} mean abs {mean:.3e}")
    if w.dtype == "bf16":
        assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS
    else:
        assert mx <= gu.F32_MAX_ABS


def test_attention_strided_layout_and_batch():
    """[b, L, H, d] storage and batch 2 through the MFMA kernel."""
    ws = [ri.custom(L=512, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=s, logit_gain=2.0) for s in (51, 52)]
    xs = [ri.generate(w) for w in ws]
    dev = [gu.to_device(x, "bf16") for x in xs]
    cat = {k: torch.cat([d[k] for d in dev], 0) for k in "QKV"}
    cat = {k: v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for k, v in cat.items()}
    p = rr()
    mask = p.rr_estimate(cat["Q"], cat["K"], 16, 128, 0.9)
    O = p.rr_sparse_attn(cat["Q"], cat["K"], cat["V"], mask)
    torch.cuda.synchronize()
    assert O.stride() == cat["Q"].stride()
    dense = mask.dense.cpu().numpy()
    for b, x in enumerate(xs):
        O_ref, _ = oracle.sparse_attention(x["Q"], x["K"], x["V"], dense[b], 128)
        mx, mean = gu.attention_errors(O[b], O_ref)
        _say(f"[attn] strided batch {b}: max abs {mx:.3e} mean abs {mean:.3e}")
        assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS


def test_row_order_is_a_sorted_permutation_and_changes_no_result():
    """The scheduling hint lists every row of a KV head once, heaviest first (ties by row id); the
    attention output does not depend on it."""
    import dataclasses
    w = ri.custom(L=4096, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=51, logit_gain=3.0)
    t = gu.to_device(ri.generate(w), w.dtype)
    p = rr()
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.85)
    torch.cuda.synchronize()
    assert mask.row_order is not None and mask.row_order.shape == (1, w.Hkv, w.G * w.Nb)
    order = mask.row_order.cpu().numpy()[0]
    count = mask.row_count.cpu().numpy()[0].reshape(w.Hkv, w.G * w.Nb)
    N, G, Nb = w.G * w.Nb, w.G, w.Nb
    for kv in range(w.Hkv):
        assert np.array_equal(np.sort(order[kv]), np.arange(N))
        # the documented rule, restated: classes of 8 blocks heaviest first, then query block descending,
        # then head; launch ranks transposed inside runs of 8 G rows
        rows = np.arange(N)
        hl, m = rows // Nb, rows % Nb
        srt = np.lexsort((hl, Nb - 1 - m, (Nb - count[kv]) >> 3))
        want = np.empty(N, dtype=np.int64)
        full = N // (8 * G) * (8 * G)
        for i, row in enumerate(srt):
            rank = i
            if i < full:
                base, wi = i // (8 * G) * (8 * G), i % (8 * G)
                rank = base + 8 * (wi % G) + wi // G
            want[rank] = row
        assert np.array_equal(order[kv], want)
    O1 = p.rr_sparse_attn(t["Q"], t["K"], t["V"], mask)
    O2 = p.rr_sparse_attn(t["Q"], t["K"], t["V"], dataclasses.replace(mask, row_order=None))
    torch.cuda.synchronize()
    assert torch.equal(O1, O2)
    # a hint with rows left out or out of range: those rows are skipped, nothing faults
    bad = mask.row_order.clone()
    bad[0, 0, :5] = -1
    bad[0, 1, :5] = w.G * w.Nb
    O3 = torch.zeros_like(O1)
    p.rr_sparse_attn(t["Q"], t["K"], t["V"], dataclasses.replace(mask, row_order=bad), O=O3)
    torch.cuda.synchronize()
    skipped = {(kv * w.G + int(v) // w.Nb, int(v) % w.Nb) for kv in range(w.Hkv) for v in order[kv][:5]}
    for h in range(w.Hq):
        for m in range(w.Nb):
            blk = O3[0, h, m * w.B:(m + 1) * w.B]
            if (h, m) in skipped:
                assert bool((blk == 0).all())
            else:
                assert torch.equal(blk, O1[0, h, m * w.B:(m + 1) * w.B])


def test_mask_from_dense_and_padding_route():
    """rr_mask_from_dense against the host-built lists; and the route for a length that is not a multiple
    of B: pad Q, K, V at the end -- causality keeps every real row independent of what the padding holds."""
    w = ri.custom(L=2048, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=81, logit_gain=3.0)
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    p = rr()
    rng = np.random.default_rng(5)
    dense = (rng.random((w.Hq, w.Nb, w.Nb)) < 0.4).astype(np.uint8) * 7          # any nonzero byte selects
    dense[1, 5, :] = 0                                                             # an empty row
    want = gu.blockmask_from_dense(np.tril(dense != 0).astype(np.uint8), w.B)
    got = p.rr_mask_from_dense(t["Q"], t["K"], torch.from_numpy(dense)[None].to("cuda:0"), w.B)
    torch.cuda.synchronize()
    assert torch.equal(got.row_count, want.row_count)
    cnt = want.row_count.cpu().numpy()[0]
    gl, wl = got.row_list.cpu().numpy()[0], want.row_list.cpu().numpy()[0]
    for h in range(w.Hq):
        for m in range(w.Nb):
            assert np.array_equal(gl[h, m, :cnt[h, m]], wl[h, m, :cnt[h, m]])
    order = got.row_order.cpu().numpy()[0]
    for kv in range(w.Hkv):
        assert np.array_equal(np.sort(order[kv]), np.arange(w.G * w.Nb))
    O1 = p.rr_sparse_attn(t["Q"], t["K"], t["V"], got)
    O2 = p.rr_sparse_attn(t["Q"], t["K"], t["V"], want)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2)

    # real length 1900, padded to the next multiple of B (1920): two different paddings, same results
    # on the real rows (the partly padded last query block is the protected one and keeps every block)
    Lr, Lp = 1900, 1920
    outs = []
    for fill in (0.0, 3.0):
        Q, K, V = (t[k][:, :, :Lp].contiguous() for k in "QKV")
        for z in (Q, K, V):
            z[:, :, Lr:, :] = fill
        mask = p.rr_estimate(Q, K, w.S, w.B, 0.85)
        O = p.rr_sparse_attn(Q, K, V, mask)
        torch.cuda.synchronize()
        outs.append((mask.dense.clone(), O[:, :, :Lr].clone()))
    assert torch.equal(outs[0][0], outs[1][0])
    assert bool(torch.tril(outs[0][0][0, 0])[Lp // w.B - 1].all())
    # same values up to bf16 rounding: a wave moves its lazy softmax reference when ANY of its queries
    # needs it, so what the padded queries of a wave hold can change the rounding of P for its real ones
    diff = (outs[0][1].float() - outs[1][1].float()).abs()
    assert float(diff.max()) <= 1e-2 and float(diff.mean()) <= 1e-4


def test_malformed_lists_are_clamped_not_followed():
    """Counts and entries outside their ranges (caller-made lists) are clamped on the device."""
    import dataclasses
    for d, B, dtype in ((128, 128, "bf16"), (64, 64, "f32")):
        w = ri.custom(L=16 * B, Hq=2, Hkv=1, d=d, dtype=dtype, B=B, S=B // 8, seed=95)
        t = gu.to_device(ri.generate(w), w.dtype)
        p = rr()
        dense = oracle.causal_block_mask(w.Hq, w.Nb)
        good = gu.blockmask_from_dense(dense, w.B)
        want = p.rr_sparse_attn(t["Q"], t["K"], t["V"], good)
        bad_list = good.row_list.clone()
        bad_count = good.row_count.clone()
        bad_list[0, 0, 5, 2] = 10 ** 6          # far outside: clamped to the diagonal block of row 5
        bad_list[0, 1, 7, 0] = -12345           # clamped to block 0 (which it was)
        bad_count[0, 1, 3] = 10 ** 6            # clamped to m + 1 = 4 (which it was)
        bad_count[0, 0, 9] = -4                 # clamped to 0: empty row
        got = p.rr_sparse_attn(t["Q"], t["K"], t["V"], dataclasses.replace(good, row_list=bad_list, row_count=bad_count))
        torch.cuda.synchronize()
        assert bool(torch.isfinite(got).all())
        assert torch.equal(got[0, 1], want[0, 1])
        assert bool((got[0, 0, 9 * B:10 * B] == 0).all())
        untouched = [m for m in range(w.Nb) if m not in (5, 9)]
        for m in untouched:
            assert torch.equal(got[0, 0, m * B:(m + 1) * B], want[0, 0, m * B:(m + 1) * B])


@pytest.mark.parametrize("form", ["plain", "packed_ragged", "many_rows", "decode_step", "chunk_with_workspace"])
def test_path_is_capturable_in_a_hip_graph(form):
    """The library only enqueues kernels on the caller's stream (no allocation, no memset, no sync), so
    estimate + sparse attention can be captured once and replayed; every replay is compared with the eager
    result, with other eager work and synchronisations between the replays.  Second form: packed sequences
    whose last one ends inside a block (the other instantiations of the kernels).  Third form: four times as
    many rows as compute units, so that the persistent workgroups of the sparse launch draw rows from the
    mask's queue in every replay (the launch must leave the counters at zero by itself: a captured graph has
    no clearing step).  Fourth and fifth form: the entry point with a workspace, for one new token (the decode
    kernel and its merge) and for an unaligned chunk of 1000 tokens at a 128-block context (plan kernel, attention
    with cut rows, merge): plan and partial results live in the caller's workspace and are rebuilt by every replay."""
    long_ctx = form in ("many_rows", "decode_step", "chunk_with_workspace")
    w = ri.custom(L=16384 if long_ctx else 4096, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=91,
                  logit_gain=3.0)
    t = gu.to_device(ri.generate(w), w.dtype)
    p = rr()
    sf = None
    if form == "packed_ragged":
        t = {k: v[:, :, :4096 - 55].contiguous() for k, v in t.items()}
        sf = p.packed_seq_first([7, 1, 24], "cuda:0")
    Q, K, V = t["Q"], t["K"], t["V"]
    rows, wa, flags = w.Nb, None, 1
    if form in ("decode_step", "chunk_with_workspace"):
        q0 = w.L - (1 if form == "decode_step" else 1000)
        Q = Q[:, :, q0:].contiguous()
        rows, flags = w.Nb - q0 // w.B, 0
        need = p.rr_attn_workspace_bytes(Q, K, w.B)
        assert need > 0
        wa = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    ws = torch.empty(p.rr_workspace_bytes(Q, K, w.S, w.B), dtype=torch.uint8, device="cuda:0")
    mask = p.BlockMask.allocate(1, w.Hq, w.Nb, w.B, "cuda:0", dense=True, Hkv=w.Hkv, rows=rows)
    O = torch.empty_like(Q)

    def step():
        p.rr_estimate(Q, K, w.S, w.B, 0.9, flags=flags, out=mask, workspace=ws, seq_first=sf)
        p.rr_sparse_attn(Q, K, V, mask, O=O, workspace=wa)

    step()
    torch.cuda.synchronize()
    want_O, want_dense, want_count = O.clone(), mask.dense.clone(), mask.row_count.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()                                          # warm-up on the capture stream
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for replay in range(3):
        O.fill_(float("nan"))
        mask.dense.zero_()
        mask.row_count.zero_()
        if wa is not None:
            wa.fill_(0xFF)                              # plan and partial results of the previous replay are gone
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want_O) and torch.equal(mask.dense, want_dense), replay
        assert torch.equal(mask.row_count, want_count), replay
        assert int(mask.queue.abs().sum().item()) == 0, replay
        (K[:, :, :4096].float() @ K[:, :, :4096].float().transpose(-1, -2)[..., :64]).sum().item()   # unrelated eager work in between


def test_end_to_end_tau_one_equals_dense():
    """tau = 1 keeps every causal block, so estimate + sparse attention is dense attention."""
    w = ri.custom(L=1024, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=61)
    t = gu.to_device(ri.generate(w), "bf16")
    p = rr()
    mask = p.rr_estimate(t["Q"], t["K"], 16, 128, 1.0)
    O = p.rr_sparse_attn(t["Q"], t["K"], t["V"], mask)
    Od = p.rr_dense_attn(t["Q"], t["K"], t["V"], 128)
    torch.cuda.synchronize()
    assert torch.equal(O, Od)


CHUNK_CASES = {
    # name: (workload, first token of the chunk, tau)
    "mfma_last_quarter": (ri.custom(L=4096, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=101, logit_gain=3.0), 3072, 0.85),
    "mfma_single_block_S8": (ri.custom(L=2048, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=8, seed=102, logit_gain=2.5), 1920, 0.9),
    "mfma_mid_G7": (ri.custom(L=1536, Hq=7, Hkv=1, d=128, dtype="bf16", B=128, S=32, seed=103, logit_gain=2.5), 640, 0.9),
    "generic_f32": (ri.custom(L=1024, Hq=4, Hkv=2, d=64, dtype="f32", B=64, S=8, seed=104, logit_gain=2.5), 448, 0.8),
    "generic_bf16_B32": (ri.custom(L=768, Hq=6, Hkv=3, d=96, dtype="bf16", B=32, S=4, seed=105, logit_gain=2.0), 512, 0.9),
}


@pytest.mark.parametrize("name", list(CHUNK_CASES))
def test_chunked_prefill_matches_the_rows_of_the_full_computation(name):
    """Chunked prefill: Q holds the last Lq positions of the context.  Masks, outputs, lse, the row order and
    the accuracy diagnostic of the chunk must be the corresponding rows of the oracle's full-sequence result
    (last-query-block protection on: the chunk ends the sequence)."""
    w, q0, tau = CHUNK_CASES[name]
    _say(f"[chunk] case={name} L={w.L} q0={q0} Hq={w.Hq} d={w.d} {w.dtype} B={w.B} S={w.S} tau={tau}")
    x = ri.generate(w)
    ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, w.S, w.B, tau, True)
    m0 = q0 // w.B
    t = gu.to_device(x, w.dtype)
    Qc = t["Q"][:, :, q0:, :]                               # a view: rows q0 .. L-1, strides of the full tensor
    p = rr()
    mask = p.rr_estimate(Qc, t["K"], w.S, w.B, tau, block_mass=True)
    torch.cuda.synchronize()
    rows = w.Nb - m0
    assert mask.dense.shape == (1, w.Hq, rows, w.Nb) and mask.row_count.shape == (1, w.Hq, rows)
    dense = mask.dense.cpu().numpy()[0]
    rep = oracle.compare_masks(ref_mask[:, m0:], ref_margin[:, m0:], ref_frac[:, m0:], dense, margin_tol=gu.MARGIN_TOL)
    _say(f"[chunk] {name}: {rep}")
    assert rep["failed"] == 0
    assert np.abs(mask.block_mass.cpu().numpy()[0] - ref_frac[:, m0:]).max() < 2e-5
    count, lst = mask.row_count.cpu().numpy()[0], mask.row_list.cpu().numpy()[0]
    for h in range(w.Hq):
        for r in range(rows):
            assert np.array_equal(lst[h, r, :count[h, r]], np.nonzero(dense[h, r])[0])
    order = mask.row_order.cpu().numpy()[0]
    for kv in range(w.Hkv):
        assert np.array_equal(np.sort(order[kv]), np.arange(w.G * rows))

    lse = torch.empty((1, w.Hq, w.L - q0), dtype=torch.float32, device="cuda:0")
    O = p.rr_sparse_attn(Qc, t["K"], t["V"], mask, lse=lse)
    Od = p.rr_dense_attn(Qc, t["K"], t["V"], w.B)
    torch.cuda.synchronize()
    full_mask = np.zeros((w.Hq, w.Nb, w.Nb), dtype=np.uint8)
    full_mask[:, m0:] = dense
    full_mask[:, :m0] = oracle.causal_block_mask(w.Hq, w.Nb)[:, :m0]
    O_ref, lse_ref = oracle.sparse_attention(x["Q"], x["K"], x["V"], full_mask, w.B)
    Od_ref, _ = oracle.dense_attention(x["Q"], x["K"], x["V"], w.B)
    for label, got, ref in (("sparse", O, O_ref), ("dense", Od, Od_ref)):
        mx, mean = gu.attention_errors(got[0], ref[:, q0:])
        _say(f"[chunk] {name} {label}: max abs {mx:.3e} mean abs {mean:.3e}")
        if w.dtype == "bf16":
            assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS
        else:
            assert mx <= gu.F32_MAX_ABS
    assert np.abs(lse[0].cpu().numpy() - lse_ref[:, q0:]).max() < (2e-2 if w.dtype == "bf16" else 1e-4)

    # caller-made mask and the accuracy diagnostic on the chunk
    again = p.rr_mask_from_dense(Qc, t["K"], mask.dense, w.B)
    torch.cuda.synchronize()
    assert torch.equal(again.row_count, mask.row_count)
    acc = p.rr_selection_accuracy(Qc, t["K"], mask, 0.95, step=w.B // 2).cpu().numpy()[0]
    G = w.G
    for h in (0, w.Hq - 1):
        ps = rs = 0.0
        qs = list(range(q0 + w.B // 2 - 1, w.L, w.B // 2))
        for i in qs:
            inter, pred, star = oracle.selection_accuracy_query(x["Q"][h], x["K"][h // G], full_mask[h, i // w.B], i, w.B, 0.95)
            ps += inter / pred if pred else 0.0
            rs += inter / star
        assert abs(acc[h, 0] - ps / len(qs)) <= 2e-3 and abs(acc[h, 1] - rs / len(qs)) <= 2e-3


def test_optional_outputs_may_be_absent():
    """dense, block_mass and row_order are optional: without them the required count / list are unchanged."""
    w = ri.custom(L=2048, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=111, logit_gain=3.0)
    t = gu.to_device(ri.generate(w), w.dtype)
    p = rr()
    full = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.85, block_mass=True)
    bare = p.BlockMask.allocate(1, w.Hq, w.Nb, w.B, "cuda:0", dense=False)
    p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.85, out=bare)
    torch.cuda.synchronize()
    assert bare.dense is None and bare.block_mass is None and bare.row_order is None
    assert torch.equal(bare.row_count, full.row_count)
    cnt = full.row_count.cpu().numpy()[0]
    a, b = bare.row_list.cpu().numpy()[0], full.row_list.cpu().numpy()[0]
    for h in range(w.Hq):
        for m in range(w.Nb):
            assert np.array_equal(a[h, m, :cnt[h, m]], b[h, m, :cnt[h, m]])
    O1 = p.rr_sparse_attn(t["Q"], t["K"], t["V"], bare)
    O2 = p.rr_sparse_attn(t["Q"], t["K"], t["V"], full)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2)


@pytest.mark.parametrize("scale_q,scale_k", [(6.0, 1.0), (0.02, 0.02), (3.0, 3.0)])
def test_extreme_logit_ranges(scale_q, scale_k):
    """Saturated softmax (logits of +-100 and more: the lazy reference of the attention kernel moves often, one
    key dominates a row), and nearly flat softmax (tiny logits)."""
    w = ri.custom(L=2048, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=121, logit_gain=2.0)
    x = ri.generate(w)
    x = {"Q": ri.bf16_round(x["Q"] * scale_q), "K": ri.bf16_round(x["K"] * scale_k), "V": x["V"]}
    t = gu.to_device(x, w.dtype)
    p = rr()
    ref_mask, ref_frac, ref_margin = gu.oracle_estimate(x, w.S, w.B, 0.9, True)
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9, block_mass=True)
    torch.cuda.synchronize()
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, 0.9)
    _say(f"[extreme] q x{scale_q} k x{scale_k}: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 5e-5
    lse = torch.empty((1, w.Hq, w.L), dtype=torch.float32, device="cuda:0")
    O = p.rr_sparse_attn(t["Q"], t["K"], t["V"], mask, lse=lse)
    Od = p.rr_dense_attn(t["Q"], t["K"], t["V"], w.B)
    torch.cuda.synchronize()
    got = mask.dense.cpu().numpy()[0]
    O_ref, lse_ref = oracle.sparse_attention(x["Q"], x["K"], x["V"], got, w.B)
    Od_ref, _ = oracle.dense_attention(x["Q"], x["K"], x["V"], w.B)
    for label, a, b in (("sparse", O, O_ref), ("dense", Od, Od_ref)):
        mx, mean = gu.attention_errors(a[0], b)
        _say(f"[extreme] {label}: max abs {mx:.3e} mean abs {mean:.3e}")
        assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS
    assert np.abs(lse[0].cpu().numpy() - lse_ref).max() < 2e-2 * max(1.0, scale_q * scale_k)


def test_attention_is_deterministic_over_many_launches():
    """No atomics, no run-to-run ordering effects: 20 launches of sparse and dense attention, bit-identical."""
    w = ri.custom(L=8192, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=131, logit_gain=3.0)
    t = gu.to_device(ri.generate(w), w.dtype)
    p = rr()
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9)
    O0 = p.rr_sparse_attn(t["Q"], t["K"], t["V"], mask)
    D0 = p.rr_dense_attn(t["Q"], t["K"], t["V"], w.B)
    torch.cuda.synchronize()
    for k in range(20):
        O = p.rr_sparse_attn(t["Q"], t["K"], t["V"], mask)
        D = p.rr_dense_attn(t["Q"], t["K"], t["V"], w.B)
        m2 = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9)
        torch.cuda.synchronize()
        assert torch.equal(O, O0) and torch.equal(D, D0), k
        assert torch.equal(m2.dense, mask.dense) and torch.equal(m2.row_order, mask.row_order), k
