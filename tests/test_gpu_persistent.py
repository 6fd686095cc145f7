"""rr_sparse_attn with a row queue (persistent workgroups that draw rows from per-XCD counters) against the
same launch without one (a workgroup per row): the same per-row arithmetic, so every result is equal bit for
bit.  The oracle comparison of both is in the parity tests; here the scheduling is what is tested: more rows
than workgroups, rows left out of the order, lengths that end inside a block, steps, repeated launches."""
import dataclasses

import numpy as np
import pytest
import torch

import rr_inputs as ri
import gpu_util as gu

pytestmark = pytest.mark.gpu


def rr():
    import paper_2602_05853_amd as p
    return p


def _both(p, t, mask, L=None, Lq=None):
    """O and lse with the queue and without it."""
    Q = t["Q"]
    out = []
    for m in (mask, dataclasses.replace(mask, queue=None)):
        O = torch.full_like(Q, float("nan"))
        lse = torch.full((Q.shape[0], Q.shape[1], Q.shape[2]), float("nan"), dtype=torch.float32, device=Q.device)
        p.rr_sparse_attn(Q, t["K"], t["V"], m, O=O, lse=lse)
        torch.cuda.synchronize()
        out.append((O, lse))
    return out


@pytest.mark.parametrize("L,Hq,Hkv,tau", [(16384, 8, 2, 0.85), (16384 - 37, 8, 2, 0.9), (8192, 32, 8, 0.95),
                                          (2048, 4, 4, 0.9)])
def test_queue_launch_equals_row_per_workgroup_launch(L, Hq, Hkv, tau):
    p = rr()
    w = ri.custom(L=L, Hq=Hq, Hkv=Hkv, d=128, dtype="bf16", B=128, S=16, seed=77, logit_gain=3.0)
    t = gu.to_device(ri.generate(w), w.dtype)
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, tau)
    torch.cuda.synchronize()
    assert mask.queue is not None and mask.queue.numel() == p.binding.RR_QUEUE_WORDS
    assert int(mask.queue.abs().sum().item()) == 0
    print(f"[persistent] L={L} {Hq}/{Hkv} heads: {Hq * ((L + 127) // 128)} rows", flush=True)
    for rep in range(3):                                    # the launch leaves the queue ready for the next one
        (O1, l1), (O2, l2) = _both(p, t, mask)
        assert int(mask.queue.abs().sum().item()) == 0, rep
        assert not torch.isnan(O1).any() and not torch.isnan(l1).any()
        assert torch.equal(O1, O2) and torch.equal(l1, l2), rep


def test_queue_launch_skips_rows_left_out_of_the_order():
    p = rr()
    w = ri.custom(L=8192, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=78, logit_gain=3.0)
    t = gu.to_device(ri.generate(w), w.dtype)
    mask = p.rr_estimate(t["Q"], t["K"], w.S, w.B, 0.9)
    torch.cuda.synchronize()
    order = mask.row_order.cpu().numpy()[0]
    bad = mask.row_order.clone()
    bad[0, 0, 3:40] = -1
    bad[0, 1, 100:130] = w.G * w.Nb
    O = torch.zeros_like(t["Q"])
    p.rr_sparse_attn(t["Q"], t["K"], t["V"], dataclasses.replace(mask, row_order=bad), O=O)
    torch.cuda.synchronize()
    assert int(mask.queue.abs().sum().item()) == 0
    ref = p.rr_sparse_attn(t["Q"], t["K"], t["V"], dataclasses.replace(mask, queue=None))
    torch.cuda.synchronize()
    skipped = {(0 * w.G + int(v) // w.Nb, int(v) % w.Nb) for v in order[0][3:40]}
    skipped |= {(1 * w.G + int(v) // w.Nb, int(v) % w.Nb) for v in order[1][100:130]}
    for h in range(w.Hq):
        for m in range(w.Nb):
            blk = O[0, h, m * w.B:(m + 1) * w.B]
            if (h, m) in skipped:
                assert bool((blk == 0).all()), (h, m)
            else:
                assert torch.equal(blk, ref[0, h, m * w.B:(m + 1) * w.B]), (h, m)


def test_queue_launch_on_a_step_that_starts_inside_a_block():
    p = rr()
    w = ri.custom(L=8192, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, seed=79, logit_gain=3.0)
    t = gu.to_device(ri.generate(w), w.dtype)
    q0 = 8192 - 3000 - 45
    ts = {"Q": t["Q"][:, :, q0:].contiguous(), "K": t["K"], "V": t["V"]}
    mask = p.rr_estimate(ts["Q"], ts["K"], w.S, w.B, 0.9, flags=0)
    torch.cuda.synchronize()
    (O1, l1), (O2, l2) = _both(p, ts, mask)
    assert int(mask.queue.abs().sum().item()) == 0
    assert not torch.isnan(O1).any() and not torch.isnan(l1).any()
    assert torch.equal(O1, O2) and torch.equal(l1, l2)
