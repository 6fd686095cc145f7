"""The seeded input generator: determinism, value grid, and that the structure it plants is there."""
import math

import numpy as np

import rr_inputs as ri


def test_deterministic_and_thread_independent():
    w = ri.custom(L=2048, Hq=4, Hkv=2, d=64, dtype="bf16", B=64, S=8, seed=7, n_spans=2, logit_gain=2.0)
    a = ri.generate(w, threads=1)
    b = ri.generate(w, threads=4)
    for k in "QKV":
        assert np.array_equal(a[k], b[k])
    c = ri.generate(w.with_(seed=8), threads=4)
    assert not np.array_equal(a["Q"], c["Q"])


def test_bf16_grid_and_rounding():
    w = ri.custom(L=512, Hq=2, Hkv=1, d=64, dtype="bf16", B=64, S=8)
    x = ri.generate(w)
    for k in "QKV":
        assert (x[k].view(np.uint32) & 0xFFFF == 0).all()
        assert np.array_equal(ri.bf16_from_bits(ri.bf16_bits(x[k])), x[k])
    # ties to even on the 16 dropped bits
    v = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20], dtype=np.float32)
    assert ri.bf16_round(v).tolist() == [1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7]
    y = ri.generate(w.with_(dtype="f32"))
    assert (y["Q"].view(np.uint32) & 0xFFFF != 0).any()


def test_config_shapes():
    c = ri.CONFIGS
    assert (c["cfg0"].L, c["cfg0"].Hq, c["cfg0"].Hkv, c["cfg0"].d, c["cfg0"].B, c["cfg0"].S) == (1024, 4, 2, 64, 64, 8)
    assert (c["cfg2"].L, c["cfg2"].Hq, c["cfg2"].Hkv, c["cfg2"].d, c["cfg2"].B, c["cfg2"].S) == (131072, 32, 8, 128, 128, 16)
    assert c["cfg4"].video == (64, 1000, 1536) and sum(c["cfg4"].video[:2]) != 0
    assert c["cfg4"].video[0] * c["cfg4"].video[1] + c["cfg4"].video[2] == c["cfg4"].L
    for w in c.values():
        assert w.B % w.S == 0 and w.L % w.B == 0 and w.Hq % w.Hkv == 0


def test_planted_structure_is_measurable():
    """Mean logit boosts of the sink tokens and of the local window match their nominal values."""
    w = ri.custom(L=4096, Hq=2, Hkv=1, d=128, dtype="f32", B=128, S=16, seed=3, logit_gain=2.0)
    x = ri.generate(w)
    q, k = x["Q"][0].astype(np.float64), x["K"][0].astype(np.float64)
    logits = q[1024:] @ k.T / math.sqrt(w.d)
    base = logits[:, 512:900].mean()
    sink = logits[:, : w.sink_tokens].mean() - base
    assert abs(sink - w.sink_boost * w.logit_gain) < 0.5
    i = np.arange(1024, 4096)
    near = logits[i - 1024, i - 2].mean() - base
    far = logits[i - 1024, i - 700].mean() - base
    assert abs(near - w.window_boost * w.logit_gain) < 0.5 and abs(far) < 0.6
