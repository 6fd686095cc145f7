"""Helpers shared by the GPU parity tests: upload a workload, run the C ABI through the binding,
compare with the CPU oracle under the parity bar."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import rr_inputs as ri
from oracle import rr_oracle as oracle

BF16_MAX_ABS, BF16_MEAN_ABS = 2e-2, 2e-3     # bf16 tensors against the fp64 oracle
F32_MAX_ABS = 1e-4                           # fp32 tensors: the generic kernels keep fp32 throughout
MARGIN_TOL = 1e-4                            # a block whose decision is this close to tau may flip


def to_device(x, dtype: str, layout: str = "bhld"):
    """numpy [H, L, d] arrays -> torch [1, H, L, d] tensors on cuda:0 (optionally stored as [1, L, H, d])."""
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    out = {}
    for k in "QKV":
        t = torch.from_numpy(x[k]).to(tdt)[None].to("cuda:0")
        if layout == "blhd":
            t = t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        out[k] = t
    return out


def oracle_estimate(x, S, B, tau, protect=True, threads=8):
    Q, K = x["Q"], x["K"]
    G = Q.shape[0] // K.shape[0]
    with ThreadPoolExecutor(threads) as ex:
        outs = list(ex.map(lambda h: oracle.estimate_head(Q[h], K[h // G], h, S, B, tau, protect),
                           range(Q.shape[0])))
    return (np.stack([o[0] for o in outs]), np.stack([o[1] for o in outs]), np.stack([o[2] for o in outs]))


def check_mask_structures(mask):
    """dense / row_count / row_list of a BlockMask must describe the same selection."""
    dense = mask.dense.cpu().numpy()
    count = mask.row_count.cpu().numpy()
    lst = mask.row_list.cpu().numpy()
    assert (np.triu(dense, 1) == 0).all(), "block selected above the diagonal"
    assert np.array_equal(dense.sum(-1), count)
    b, H, Nb, _ = dense.shape
    for bi in range(b):
        for h in range(H):
            for m in range(Nb):
                want = np.nonzero(dense[bi, h, m])[0]
                assert np.array_equal(lst[bi, h, m, : count[bi, h, m]], want), (bi, h, m)
    return dense


def compare_estimate(mask, ref_mask, ref_frac, ref_margin, tau):
    dense = mask.dense.cpu().numpy()[0]
    rep = oracle.compare_masks(ref_mask, ref_margin, ref_frac, dense, margin_tol=MARGIN_TOL)
    if mask.block_mass is not None:
        bm = mask.block_mass.cpu().numpy()[0]
        rep["mass_max_abs_err"] = float(np.abs(bm - ref_frac).max())
    if rep["failed"]:
        bad = np.argwhere((dense != ref_mask).any(-1))
        rep["rows_with_mismatch"] = [(int(h), int(m), int((dense[h, m] != ref_mask[h, m]).sum()),
                                      int(dense[h, m].sum()), int(ref_mask[h, m].sum())) for h, m in bad[:8]]
    tri = np.tril(np.ones(ref_mask.shape[-2:], dtype=bool))
    rep["density"] = float(dense[:, tri].mean())
    return rep


def attention_errors(O_gpu: torch.Tensor, O_ref: np.ndarray):
    diff = np.abs(O_gpu.float().cpu().numpy().astype(np.float64) - O_ref)
    return float(diff.max()), float(diff.mean())


def blockmask_from_dense(dense_np: np.ndarray, B: int):
    """Build the device arrays of a caller-chosen 0/1 mask [H, Nb, Nb] (test helper, host side)."""
    from paper_2602_05853_amd import BlockMask
    H, Nb, _ = dense_np.shape
    count = dense_np.sum(-1).astype(np.int32)
    lst = np.zeros((H, Nb, Nb), dtype=np.int32)
    for h in range(H):
        for m in range(Nb):
            idx = np.nonzero(dense_np[h, m])[0]
            lst[h, m, : idx.size] = idx
    dev = "cuda:0"
    return BlockMask(B=B, Nb=Nb, row_count=torch.from_numpy(count)[None].to(dev),
                     row_list=torch.from_numpy(lst)[None].to(dev),
                     dense=torch.from_numpy(dense_np.astype(np.uint8))[None].to(dev))
