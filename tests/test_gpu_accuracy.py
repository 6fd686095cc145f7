"""GPU parity of the block selection accuracy diagnostic (appendix "Block Selection Accuracy Analysis")
against the fp64 oracle.  The metric counts set members decided by floating-point comparisons (is a key
among the smallest set reaching tau?), the GPU takes those decisions on fp32 attention values, so a few
positions at the boundary of K* may differ: the averaged precision / recall / F1 are compared within 2e-3
(cases without boundary effects -- exact ties, full masks -- are compared much tighter)."""
import sys

import numpy as np
import pytest
import torch

import rr_inputs as ri
from oracle import rr_oracle as oracle
import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def rr():
    import paper_2602_05853_amd as p
    return p


CASES = {
    "f32_d64": (ri.custom(L=1024, Hq=4, Hkv=2, d=64, dtype="f32", B=64, S=8, seed=71, logit_gain=2.5), 0.9, 0.95, 1),
    "bf16_d128": (ri.custom(L=2048, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=72, logit_gain=3.0), 0.8, 0.95, 1),
    "bf16_step8_tau99": (ri.custom(L=1536, Hq=2, Hkv=1, d=128, dtype="bf16", B=128, S=16, seed=73, logit_gain=3.0), 0.9, 0.99, 8),
    "f32_odd_d": (ri.custom(L=512, Hq=3, Hkv=3, d=40, dtype="f32", B=32, S=4, seed=74, logit_gain=2.0), 0.7, 0.5, 1),
}


@pytest.mark.parametrize("name", list(CASES))
def test_accuracy_of_estimated_mask_matches_oracle(name):
    w, tau_sel, tau_gt, step = CASES[name]
    _say(f"[accuracy] case={name} L={w.L} Hq={w.Hq} d={w.d} {w.dtype} B={w.B} tau_gt={tau_gt} step={step}")
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    p = rr()
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, tau_sel)
    got = p.rr_selection_accuracy(t["Q"], t["K"], mask, tau_gt, step)
    torch.cuda.synchronize()
    ref = oracle.selection_accuracy(x["Q"], x["K"], mask.dense.cpu().numpy()[0], w.B, tau_gt, step)
    err = np.abs(got[0].cpu().numpy() - ref).max()
    _say(f"[accuracy] {name}: oracle P/R/F1 head 0 {ref[0].round(4)}, max abs diff {err:.2e}")
    assert err <= TOL


def test_accuracy_special_masks_and_exact_ties():
    w = ri.custom(L=1024, Hq=2, Hkv=1, d=64, dtype="bf16", B=64, S=8, seed=75, logit_gain=2.5)
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    p = rr()
    Nb = w.Nb
    full = gu.blockmask_from_dense(oracle.causal_block_mask(w.Hq, Nb), w.B)
    got = p.rr_selection_accuracy(t["Q"], t["K"], full, 0.95).cpu().numpy()[0]
    ref = oracle.selection_accuracy(x["Q"], x["K"], oracle.causal_block_mask(w.Hq, Nb), w.B, 0.95)
    assert np.all(got[:, 1] == 1.0)                      # everything selected: recall is exactly 1
    assert np.abs(got - ref).max() <= TOL
    diag = np.broadcast_to(np.eye(Nb, dtype=np.uint8), (w.Hq, Nb, Nb)).copy()
    got = p.rr_selection_accuracy(t["Q"], t["K"], gu.blockmask_from_dense(diag, w.B), 0.95).cpu().numpy()[0]
    ref = oracle.selection_accuracy(x["Q"], x["K"], diag, w.B, 0.95)
    assert np.abs(got - ref).max() <= TOL
    empty = np.zeros_like(diag)
    empty[:, 0, 0] = 1                                   # rows with nothing selected: precision and recall 0
    got = p.rr_selection_accuracy(t["Q"], t["K"], gu.blockmask_from_dense(empty, w.B), 0.95).cpu().numpy()[0]
    ref = oracle.selection_accuracy(x["Q"], x["K"], empty, w.B, 0.95)
    assert np.abs(got - ref).max() <= TOL
    # zero queries: exactly uniform rows, every value a tie; tau = 0.73 keeps tau (i+1) off the integers
    # except at i+1 = 100, 200, ..., where fp32 and fp64 land on different sides (one position of ~100)
    Q0 = torch.zeros_like(t["Q"])
    x0 = dict(x, Q=np.zeros_like(x["Q"]))
    first = np.zeros_like(diag)
    first[:, :, 0] = 1
    for dense in (oracle.causal_block_mask(w.Hq, Nb), first, diag):
        got = p.rr_selection_accuracy(Q0, t["K"], gu.blockmask_from_dense(dense, w.B), 0.73).cpu().numpy()[0]
        ref = oracle.selection_accuracy(x0["Q"], x0["K"], dense, w.B, 0.73)
        _say(f"[accuracy] ties: got {got[0].round(5)} ref {ref[0].round(5)}")
        assert np.abs(got - ref).max() <= 1e-4


def test_accuracy_full_size_sampled():
    """cfg1 at full size, one query per block (step = B), mask from the library's own estimate."""
    w = ri.get_config("cfg1")
    x = ri.generate(w)
    t = gu.to_device(x, w.dtype)
    p = rr()
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.95)
    got = p.rr_selection_accuracy(t["Q"], t["K"], mask, 0.95, step=w.B).cpu().numpy()[0]
    torch.cuda.synchronize()
    dense = mask.dense.cpu().numpy()[0]
    heads = [0, 7, 13, 31]
    for h in heads:
        ref = oracle.selection_accuracy(x["Q"][h:h + 1], x["K"][h // w.G:h // w.G + 1], dense[h:h + 1], w.B, 0.95, step=w.B)[0]
        _say(f"[accuracy] cfg1 head {h}: got {got[h].round(4)} oracle {ref.round(4)}")
        assert np.abs(got[h] - ref).max() <= TOL
