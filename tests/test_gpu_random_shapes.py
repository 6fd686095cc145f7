"""GPU parity on seeded random shapes: every case draws dtype, head layout, d, B, S, L, tau, offset
schedule and sink / recent protection from a fixed seed, runs estimate + sparse + dense through the
C ABI and compares with the oracle under the usual bar.  Small lengths, so that the oracle takes
milliseconds and both the MFMA and the generic kernels are reached many times."""
import sys

import numpy as np
import pytest
import torch

import rr_inputs as ri
from oracle import rr_oracle as oracle
import gpu_util as gu

pytestmark = pytest.mark.gpu
N_CASES = 32


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _draw(case):
    rng = np.random.default_rng(9000 + case)
    mfma = case % 2 == 0                                   # every other case is eligible for the MFMA kernels
    if mfma:
        dtype, d, B = "bf16", 128, 128
        S = int(rng.choice([4, 8, 16, 32]))
    else:
        dtype = str(rng.choice(["bf16", "f32"]))
        d = int(rng.choice([40, 48, 64, 96, 128]))
        B = int(rng.choice([16, 32, 48, 64]))
        S = int(rng.choice([s for s in (1, 2, 3, 4, 8, 16) if B % s == 0 and B // s <= 64]))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 7] if mfma else [1, 2, 3]))
    if mfma and G * (B // S) > 256:
        G = 1
    Nb = int(rng.integers(1, 17 if mfma else 25))
    tau = float(rng.choice([0.5, 0.8, 0.9, 0.95, 1.0]))
    mode = str(rng.choice(["head", "head", "fixed", "layer", "hybrid"]))
    layer = int(rng.integers(0, 40))
    sink, recent = (int(rng.integers(0, 3)), int(rng.integers(0, 3))) if rng.random() < 0.4 else (0, 0)
    protect = bool(rng.random() < 0.8)
    w = ri.custom(L=Nb * B, Hq=Hkv * G, Hkv=Hkv, d=d, dtype=dtype, B=B, S=S, tau=tau, seed=9100 + case,
                  logit_gain=float(rng.choice([1.0, 2.5, 4.0])))
    return w, tau, mode, layer, sink, recent, protect


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_shape(case):
    import paper_2602_05853_amd as rr
    w, tau, mode, layer, sink, recent, protect = _draw(case)
    _say(f"[random] case={case} L={w.L} Hq={w.Hq} Hkv={w.Hkv} d={w.d} {w.dtype} B={w.B} S={w.S} tau={tau} {mode} "
         f"layer={layer} sink={sink} recent={recent} protect={protect}")
    x = ri.generate(w)
    G = w.G
    outs = [oracle.estimate_head(x["Q"][h], x["K"][h // G], h, w.S, w.B, tau, protect, mode, layer, sink, recent)
            for h in range(w.Hq)]
    ref_mask, ref_frac, ref_margin = (np.stack([o[i] for o in outs]) for i in range(3))
    t = gu.to_device(x, w.dtype, layout="blhd" if case % 3 == 0 else "bhld")
    mask = rr.rr_estimate(t["Q"], t["K"], w.S, w.B, tau, flags=1 if protect else 0, block_mass=True,
                          offset_mode=mode, layer=layer, sink_blocks=sink, recent_blocks=recent)
    torch.cuda.synchronize()
    gu.check_mask_structures(mask)
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
    _say(f"[random] {case}: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5

    lse = torch.empty((1, w.Hq, w.L), dtype=torch.float32, device="cuda:0")
    O = rr.rr_sparse_attn(t["Q"], t["K"], t["V"], mask, lse=lse)
    Od = rr.rr_dense_attn(t["Q"], t["K"], t["V"], w.B)
    torch.cuda.synchronize()
    got_mask = mask.dense.cpu().numpy()[0]
    O_ref, lse_ref = oracle.sparse_attention(x["Q"], x["K"], x["V"], got_mask, w.B)
    Od_ref, _ = oracle.dense_attention(x["Q"], x["K"], x["V"], w.B)
    for name, got, ref in (("sparse", O, O_ref), ("dense", Od, Od_ref)):
        mx, mean = gu.attention_errors(got[0], ref)
        if w.dtype == "bf16":
            assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS, (name, mx, mean)
        else:
            assert mx <= gu.F32_MAX_ABS, (name, mx)
    assert np.abs(lse[0].cpu().numpy() - lse_ref).max() < (2e-2 if w.dtype == "bf16" else 1e-4)


def _draw_extended(case):
    """As _draw, plus: a length that ends inside the last block, several packed sequences, the cut diagonal."""
    w, tau, mode, layer, sink, recent, protect = _draw(1000 + case)
    rng = np.random.default_rng(9500 + case)
    cut = int(rng.integers(0, w.B)) if rng.random() < 0.7 else 0          # positions missing from the last block
    L = w.L - cut
    blocks = [w.Nb]
    if w.Nb >= 2 and rng.random() < 0.6:
        k = int(rng.integers(1, min(4, w.Nb)))                             # k cuts -> k + 1 sequences
        cuts = sorted(rng.choice(np.arange(1, w.Nb), size=k, replace=False).tolist())
        blocks = [b - a for a, b in zip([0] + cuts, cuts + [w.Nb])]
    diag = bool(rng.random() < 0.5)
    return w, L, blocks, tau, mode, layer, sink, recent, protect, diag


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_shape_ragged_packed_diagonal(case):
    import paper_2602_05853_amd as rr
    w, L, blocks, tau, mode, layer, sink, recent, protect, diag = _draw_extended(case)
    _say(f"[random+] case={case} L={L} (of {w.L}) blocks={blocks} Hq={w.Hq} Hkv={w.Hkv} d={w.d} {w.dtype} B={w.B} S={w.S} "
         f"tau={tau} {mode} layer={layer} sink={sink} recent={recent} protect={protect} diagonal_token={diag}")
    x = {k: np.ascontiguousarray(v[:, :L]) for k, v in ri.generate(w).items()}
    ref_mask, ref_frac, ref_margin = oracle.estimate_packed(x["Q"], x["K"], w.S, w.B, tau, blocks, protect, mode, layer,
                                                            sink, recent, "token" if diag else "stride")
    t = gu.to_device(x, w.dtype, layout="blhd" if case % 3 == 0 else "bhld")
    sf = rr.packed_seq_first(blocks, "cuda:0") if len(blocks) > 1 else None
    flags = (rr.RR_FLAG_PROTECT_LAST if protect else 0) | (rr.RR_FLAG_DIAGONAL_TOKEN if diag else 0)
    mask = rr.rr_estimate(t["Q"], t["K"], w.S, w.B, tau, flags=flags, block_mass=True, offset_mode=mode, layer=layer,
                          sink_blocks=sink, recent_blocks=recent, seq_first=sf)
    torch.cuda.synchronize()
    gu.check_mask_structures(mask)
    rep = gu.compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau)
    _say(f"[random+] {case}: {rep}")
    assert rep["failed"] == 0 and rep["mass_max_abs_err"] < 2e-5

    lse = torch.empty((1, w.Hq, L), dtype=torch.float32, device="cuda:0")
    O = rr.rr_sparse_attn(t["Q"], t["K"], t["V"], mask, lse=lse)
    Od = rr.rr_dense_attn_packed(t["Q"], t["K"], t["V"], w.B, sf) if sf is not None else \
        rr.rr_dense_attn(t["Q"], t["K"], t["V"], w.B)
    torch.cuda.synchronize()
    got_mask = mask.dense.cpu().numpy()[0]
    O_ref, lse_ref = oracle.sparse_attention(x["Q"], x["K"], x["V"], got_mask, w.B)
    Od_ref, _ = oracle.sparse_attention(x["Q"], x["K"], x["V"], oracle.packed_causal_block_mask(w.Hq, blocks), w.B)
    for name, got, ref in (("sparse", O, O_ref), ("dense", Od, Od_ref)):
        mx, mean = gu.attention_errors(got[0], ref)
        if w.dtype == "bf16":
            assert mx <= gu.BF16_MAX_ABS and mean <= gu.BF16_MEAN_ABS, (name, mx, mean)
        else:
            assert mx <= gu.F32_MAX_ABS, (name, mx)
    empty = np.isneginf(lse_ref)
    got_lse = lse[0].cpu().numpy()
    assert np.array_equal(np.isneginf(got_lse), empty)
    assert np.abs(got_lse[~empty] - lse_ref[~empty]).max() < (2e-2 if w.dtype == "bf16" else 1e-4)
