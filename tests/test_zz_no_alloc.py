"""rr_estimate_static (the allocation-free entry point: scratch inside the library's device image) against
rr_estimate with a caller workspace.  Same kernels, so the masks must be bit-identical.  Two calls in a row, the
second on a smaller input: the shared scratch still holds the first call's contents then."""
import ctypes as C

import numpy as np
import pytest
import torch

import rr_inputs as ri
from paper_2602_05853_amd import binding as bd

pytestmark = pytest.mark.gpu


def _upload(w):
    x = ri.generate(w)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    return {k: torch.from_numpy(v).to(tdt)[None].to("cuda:0") for k, v in x.items()}


def _both(w):
    t = _upload(w)
    Q, K = t["Q"], t["K"]
    shp = bd.make_shape(Q, K)
    Nb = -(-w.L // w.B)
    need = bd.lib.rr_workspace_bytes(C.byref(shp), w.S, w.B)
    assert 0 < need <= bd.RR_STATIC_SCRATCH_BYTES
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    ref = bd.BlockMask.allocate(1, w.Hq, Nb, w.B, "cuda:0", dense=True, block_mass=True, Hkv=w.Hkv)
    got = bd.BlockMask.allocate(1, w.Hq, Nb, w.B, "cuda:0", dense=True, block_mass=True, Hkv=w.Hkv)
    cr, cg = ref.c_struct(), got.c_struct()
    stream = torch.cuda.current_stream().cuda_stream
    rc = bd.lib.rr_estimate(C.byref(shp), Q.data_ptr(), K.data_ptr(), w.S, w.B, w.tau, bd.RR_FLAG_PROTECT_LAST,
                            ws.data_ptr(), need, C.byref(cr), stream)
    assert rc == bd.RR_OK
    rc = bd.lib.rr_estimate_static(C.byref(shp), Q.data_ptr(), K.data_ptr(), w.S, w.B, w.tau,
                                   bd.RR_FLAG_PROTECT_LAST, C.byref(cg), stream)
    assert rc == bd.RR_OK
    torch.cuda.synchronize()
    cnt = ref.row_count.cpu().numpy()
    assert np.array_equal(cnt, got.row_count.cpu().numpy())
    assert np.array_equal(ref.dense.cpu().numpy(), got.dense.cpu().numpy())
    assert np.array_equal(ref.block_mass.cpu().numpy(), got.block_mass.cpu().numpy())
    assert np.array_equal(ref.row_order.cpu().numpy(), got.row_order.cpu().numpy())
    rl, gl = ref.row_list.cpu().numpy(), got.row_list.cpu().numpy()
    valid = np.arange(Nb)[None, None, None, :] < cnt[..., None]
    assert np.array_equal(rl[valid], gl[valid])
    assert cnt.sum() > 0
    return int(cnt.sum())


def test_static_scratch_entry_point_matches_rr_estimate_on_two_calls_in_a_row():
    # MFMA estimate path (bf16, d = 128), then a smaller input on the same scratch, then the generic path
    big = ri.custom(L=8192 + 128 + 48, Hq=8, Hkv=2, d=128, dtype="bf16", B=128, S=16, tau=0.9, seed=11, logit_gain=2.5)
    small = ri.custom(L=2048, Hq=4, Hkv=2, d=128, dtype="bf16", B=128, S=8, tau=0.95, seed=12, logit_gain=2.5)
    generic = ri.custom(L=1024, Hq=4, Hkv=2, d=64, dtype="f32", B=64, S=8, tau=0.9, seed=13, logit_gain=2.5)
    for w in (big, small, generic):
        assert _both(w) > 0


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    # cfg2's geometry needs far more than the library holds: refused on the host, nothing launched
    s = bd.rr_shape(1, 131072, 32, 8, 128, bd.RR_BF16, 32 * 131072 * 128, 131072 * 128, 128,
                    8 * 131072 * 128, 131072 * 128, 128, 0)
    m = bd.rr_mask(None, 0x1000, 0x1000, None, 1024, 128, None)
    assert bd.lib.rr_estimate_static(C.byref(s), 0x1000, 0x1000, 16, 128, 0.9, 1, C.byref(m), None) == bd.RR_ERR_SCRATCH_LIMIT
