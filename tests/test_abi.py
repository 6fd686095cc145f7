"""Host side of the C ABI: the library loads, exports what include/rr_attn.h declares, and turns
bad arguments into error codes before anything is launched.  No GPU is needed: every call below
fails (by design) in the host-side checks, or is a pure host computation."""
import ctypes as C
import os
import re

import pytest

from paper_2602_05853_amd import binding as bd

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "rr_attn.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rr_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert set(names) == set(bd.EXPORTS)
    for n in names:
        assert getattr(bd.lib, n) is not None


def test_header_is_plain_c_and_matches_the_binding_structs(tmp_path):
    """The header compiles as C99, and the struct layouts the ctypes binding assumes are the compiler's."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "layout.c"
    src.write_text('''
#include <stdio.h>
#include <stddef.h>
#include "rr_attn.h"
int main(void) {
    printf("%zu %zu %zu %zu\\n", sizeof(rr_shape), offsetof(rr_shape, q_stride_b), offsetof(rr_shape, kv_stride_l), offsetof(rr_shape, Lq));
    printf("%zu %zu %zu %zu\\n", sizeof(rr_mask), offsetof(rr_mask, block_mass), offsetof(rr_mask, Nb), offsetof(rr_mask, row_order));
    printf("%zu %d\\n", offsetof(rr_mask, queue), RR_QUEUE_WORDS);
    printf("%zu %zu %zu %zu\\n", sizeof(rr_estimate_opts), offsetof(rr_estimate_opts, layer), offsetof(rr_estimate_opts, recent_blocks), offsetof(rr_estimate_opts, ksum_valid));
    printf("%d %d %d %d\\n", RR_ERR_LAUNCH, RR_F32, RR_OFFSET_HYBRID, (int)RR_FLAG_PROTECT_LAST);
    return 0;
}
''')
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.dirname(HEADER), str(src), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    got = list(map(int, out))
    want = [C.sizeof(bd.rr_shape), bd.rr_shape.q_stride_b.offset, bd.rr_shape.kv_stride_l.offset, bd.rr_shape.Lq.offset,
            C.sizeof(bd.rr_mask), bd.rr_mask.block_mass.offset, bd.rr_mask.Nb.offset, bd.rr_mask.row_order.offset,
            bd.rr_mask.queue.offset, bd.RR_QUEUE_WORDS,
            C.sizeof(bd.rr_estimate_opts), bd.rr_estimate_opts.layer.offset, bd.rr_estimate_opts.recent_blocks.offset,
            bd.rr_estimate_opts.ksum_valid.offset,
            bd.RR_ERR_LAUNCH, bd.RR_F32, bd.RR_OFFSET_HYBRID, bd.RR_FLAG_PROTECT_LAST]
    assert got == want


def test_version_and_status_strings():
    assert bd.lib.rr_version() >= 100
    for code in range(-7, 1):
        assert bd.lib.rr_status_string(code)
    assert bd.lib.rr_status_string(-99) == b"unknown status"


def shape(L=1024, Hq=4, Hkv=2, d=64, dtype=bd.RR_F32, batch=1):
    return bd.rr_shape(batch, L, Hq, Hkv, d, dtype, Hq * L * d, L * d, d, Hkv * L * d, L * d, d)


def test_workspace_bytes_formula():
    s = shape(L=1024, Hkv=2, d=64)
    # stride sums of K in fp32: Hkv * (L/S) * d * 4 bytes; the softmax state fits in LDS here
    assert bd.lib.rr_workspace_bytes(C.byref(s), 8, 64) == 2 * 128 * 64 * 4
    assert bd.lib.rr_workspace_bytes(C.byref(s), 7, 64) == 0          # S does not divide B
    # B need not divide L: 1024 positions are 11 blocks of 96 (the last partial), 132 strides of 8 with the filler
    assert bd.lib.rr_workspace_bytes(C.byref(s), 8, 96) == 2 * 132 * 64 * 4
    big = shape(L=131072, Hq=32, Hkv=8, d=128, dtype=bd.RR_BF16)
    # MFMA estimate path: three bf16 planes of stride sums + one fp32 block mass per (head, query block, key block):
    # 176 MiB at 128K tokens
    assert bd.lib.rr_workspace_bytes(C.byref(big), 16, 128) == 3 * 8 * 8192 * 128 * 2 + 32 * 1024 * 1024 * 4
    assert bd.lib.rr_workspace_bytes(C.byref(big), 16, 128) <= 256 << 20


FAKE = 0x1000  # a non-NULL, 16-byte aligned value; never dereferenced because the checks fail first


def call_estimate(s, Q=FAKE, K=FAKE, S=8, B=64, tau=0.9, flags=1, ws=FAKE * 16, ws_bytes=1 << 30, mask=None):
    m = mask if mask is not None else bd.rr_mask(None, FAKE, FAKE, None, s.L // B if B and s.L % B == 0 else 0, B)
    return bd.lib.rr_estimate(C.byref(s), Q, K, S, B, tau, flags, ws, ws_bytes, C.byref(m), None)


def test_estimate_ex_argument_errors():
    s = shape()
    m = bd.rr_mask(None, FAKE, FAKE, None, 16, 64, None)

    def call(opts):
        return bd.lib.rr_estimate_ex(C.byref(s), FAKE, FAKE, 8, 64, 0.9, opts, FAKE * 16, 1 << 30, C.byref(m), None)
    assert call(None) == bd.RR_ERR_NULL
    assert call(C.byref(bd.rr_estimate_opts(1, 4, 0, 0, 0))) == bd.RR_ERR_PARAM       # unknown offset mode
    assert call(C.byref(bd.rr_estimate_opts(1, -1, 0, 0, 0))) == bd.RR_ERR_PARAM
    assert call(C.byref(bd.rr_estimate_opts(1, 2, -3, 0, 0))) == bd.RR_ERR_PARAM      # negative layer
    assert call(C.byref(bd.rr_estimate_opts(1, 0, 0, -1, 0))) == bd.RR_ERR_PARAM
    assert call(C.byref(bd.rr_estimate_opts(1, 0, 0, 0, -1))) == bd.RR_ERR_PARAM
    assert call(C.byref(bd.rr_estimate_opts(8, 0, 0, 0, 0))) == bd.RR_ERR_PARAM       # unknown flag
    # stride sums kept from call to call: a capacity below L or off the block grid, more valid positions than there are
    assert call(C.byref(bd.rr_estimate_opts(1, 0, 0, 0, 0, None, 512, 0))) == bd.RR_ERR_PARAM
    assert call(C.byref(bd.rr_estimate_opts(1, 0, 0, 0, 0, None, 2048 + 8, 0))) == bd.RR_ERR_PARAM
    assert call(C.byref(bd.rr_estimate_opts(1, 0, 0, 0, 0, None, 2048, 1025))) == bd.RR_ERR_PARAM
    assert call(C.byref(bd.rr_estimate_opts(1, 0, 0, 0, 0, None, 0, 64))) == bd.RR_ERR_PARAM


def test_chunked_prefill_shape_checks():
    """Lq: 0 or L = ordinary prefill; 0 < Lq < L = the last Lq queries, at any offset."""
    s = shape()
    m = bd.rr_mask(None, FAKE, FAKE, None, 16, 64, None)

    def est(Lq):
        s.Lq = Lq
        return bd.lib.rr_estimate(C.byref(s), FAKE, FAKE, 8, 64, 0.9, 1, None, 0, C.byref(m), None)
    assert est(0) == bd.RR_ERR_WORKSPACE and est(1024) == bd.RR_ERR_WORKSPACE and est(256) == bd.RR_ERR_WORKSPACE
    assert est(2048) == bd.RR_ERR_SHAPE and est(-64) == bd.RR_ERR_SHAPE        # more queries than keys
    # a step may start anywhere (decode stage): 100 or 1 queries pass the shape checks like any other count
    assert est(100) == bd.RR_ERR_WORKSPACE and est(1) == bd.RR_ERR_WORKSPACE
    s.Lq = 96
    assert bd.lib.rr_dense_attn(C.byref(s), FAKE, FAKE, FAKE, 64, None, None, None) == bd.RR_ERR_NULL
    # the MFMA estimate workspace shrinks with the number of query blocks
    big = shape(L=131072, Hq=32, Hkv=8, d=128, dtype=bd.RR_BF16)
    big.Lq = 8192
    # ... and with only 64 workgroups the key tiles are split 12 ways: one (reference, sum) pair per chunk and
    # sampled-query slot on top
    assert bd.lib.rr_workspace_bytes(C.byref(big), 16, 128) == 3 * 8 * 8192 * 128 * 2 + 32 * 64 * 1024 * 4 + \
        8 * 8 * 12 * 256 * 8
    # attention with a workspace: nothing for a prefill; a one-token step at 128K runs on the decode kernel, 64 parts
    # per KV head (512 workgroups in all), one fp32 output row and one lse per part and query row; a 16-token step
    # on the matrix kernel with its 32 rows split 16 ways
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 128) == 0 or big.Lq != 0
    big.Lq = 0
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 128) == 0
    big.Lq = 1
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 128) == 64 * 32 * 1 * (128 * 4 + 4)
    big.Lq = 2
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 128) == 64 * 32 * 2 * (128 * 4 + 4)
    big.Lq = 16
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 128) == 16 * 32 * 16 * (128 * 4 + 4)
    # a chunk of 1024 tokens at 128K (256 rows): a plan (header, one word per row, one per slot, one per cut row) and 1024 slots of one
    # fp32 tile and its 128 lse values for the parts of the rows that are cut
    big.Lq = 1024
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 128) == 256 + 256 * 4 + 1024 * 4 + 512 * 4 + 1024 * 128 * 4 + 1024 * 128 * 128 * 4
    # ... 8192 tokens: 2048 rows, 2048 slots; 16384 tokens: 4096 rows, parts of 128 entries; 32768 tokens: too many rows to gain from it
    big.Lq = 8192
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 128) == 256 + 2048 * 4 + 2048 * 4 + 1024 * 4 + 2048 * 128 * 4 + 2048 * 128 * 128 * 4
    big.Lq = 32768
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 128) == 0
    big.Lq = 1
    assert bd.lib.rr_attn_workspace_bytes(C.byref(big), 64) == 0       # B = 64: the generic kernel, never split
    assert bd.lib.rr_dense_attn_ws(C.byref(big), FAKE, FAKE, FAKE, 128, FAKE, None, FAKE, 16, None) == bd.RR_ERR_WORKSPACE
    s.Lq = 512
    assert bd.lib.rr_accuracy_workspace_bytes(C.byref(s), 4) == s.batch * s.Hq * (512 // 4) * (s.L * 4 + 8)


def test_selection_accuracy_argument_errors():
    s = shape()
    m = bd.rr_mask(None, FAKE, FAKE, None, 16, 64, None)

    def call(tau=0.95, step=1, mask=m, out=FAKE, ws=FAKE * 16, ws_bytes=1 << 40):
        return bd.lib.rr_selection_accuracy(C.byref(s), FAKE, FAKE, C.byref(mask) if mask else None, tau, step, ws,
                                            ws_bytes, out, None)
    assert call(tau=1.0) == bd.RR_ERR_PARAM and call(tau=0.0) == bd.RR_ERR_PARAM
    assert call(step=0) == bd.RR_ERR_PARAM and call(step=3) == bd.RR_ERR_PARAM      # step must divide L
    assert call(mask=None) == bd.RR_ERR_NULL and call(out=None) == bd.RR_ERR_NULL
    assert call(mask=bd.rr_mask(None, FAKE, FAKE, None, 8, 64, None)) == bd.RR_ERR_PARAM
    assert call(ws_bytes=16) == bd.RR_ERR_WORKSPACE and call(ws=None) == bd.RR_ERR_WORKSPACE
    # one fp32 row of L per sampled query + (precision, recall) per sampled query
    assert bd.lib.rr_accuracy_workspace_bytes(C.byref(s), 4) == s.batch * s.Hq * (s.L // 4) * (s.L * 4 + 8)
    assert bd.lib.rr_accuracy_workspace_bytes(C.byref(s), 3) == 0


def test_estimate_argument_errors():
    s = shape()
    assert call_estimate(s, Q=None) == bd.RR_ERR_NULL
    assert call_estimate(s, K=None) == bd.RR_ERR_NULL
    assert call_estimate(s, mask=bd.rr_mask(None, None, FAKE, None, 16, 64)) == bd.RR_ERR_NULL
    assert call_estimate(s, S=7) == bd.RR_ERR_SHAPE
    assert call_estimate(s, B=96) == bd.RR_ERR_PARAM                              # 11 blocks of 96, the mask says 16
    assert call_estimate(s, B=96, mask=bd.rr_mask(None, FAKE, FAKE, None, 11, 96), ws=None) == bd.RR_ERR_WORKSPACE
    assert call_estimate(s, B=136) == bd.RR_ERR_SHAPE                             # B > 128
    assert call_estimate(s, tau=0.0) == bd.RR_ERR_PARAM
    assert call_estimate(s, tau=1.5) == bd.RR_ERR_PARAM
    assert call_estimate(s, tau=float("nan")) == bd.RR_ERR_PARAM
    assert call_estimate(s, flags=4) == bd.RR_ERR_PARAM
    assert call_estimate(s, mask=bd.rr_mask(None, FAKE, FAKE, None, 15, 64)) == bd.RR_ERR_PARAM
    assert call_estimate(s, ws=None) == bd.RR_ERR_WORKSPACE
    assert call_estimate(s, ws_bytes=16) == bd.RR_ERR_WORKSPACE
    assert call_estimate(s, ws=FAKE * 16 + 64) == bd.RR_ERR_WORKSPACE            # not 256-byte aligned
    assert call_estimate(s, Q=FAKE + 4) == bd.RR_ERR_SHAPE                        # misaligned rows
    assert call_estimate(shape(dtype=7)) == bd.RR_ERR_DTYPE
    assert call_estimate(shape(Hq=5, Hkv=2)) == bd.RR_ERR_SHAPE
    assert call_estimate(shape(d=60)) == bd.RR_ERR_SHAPE
    bad = shape()
    bad.q_stride_l = 66                                                           # not a multiple of 16 bytes
    assert call_estimate(bad) == bd.RR_ERR_SHAPE
    assert bd.lib.rr_estimate(None, FAKE, FAKE, 8, 64, 0.9, 1, FAKE, 1 << 30, None, None) == bd.RR_ERR_NULL


def test_attention_argument_errors():
    s = shape()
    m = bd.rr_mask(None, FAKE, FAKE, None, 16, 64)
    assert bd.lib.rr_sparse_attn(C.byref(s), None, FAKE, FAKE, C.byref(m), FAKE, None, None) == bd.RR_ERR_NULL
    assert bd.lib.rr_sparse_attn(C.byref(s), FAKE, FAKE, FAKE, None, FAKE, None, None) == bd.RR_ERR_NULL
    wrong = bd.rr_mask(None, FAKE, FAKE, None, 8, 64)
    assert bd.lib.rr_sparse_attn(C.byref(s), FAKE, FAKE, FAKE, C.byref(wrong), FAKE, None, None) == bd.RR_ERR_PARAM
    assert bd.lib.rr_dense_attn(C.byref(s), FAKE, FAKE, FAKE, 136, FAKE, None, None) == bd.RR_ERR_SHAPE      # B > 128
    assert bd.lib.rr_dense_attn(C.byref(s), FAKE, FAKE, None, 64, FAKE, None, None) == bd.RR_ERR_NULL
    chunk = shape()
    chunk.Lq = 1000                                                    # a step and packed sequences do not combine
    assert bd.lib.rr_dense_attn_packed(C.byref(chunk), FAKE, FAKE, FAKE, 64, FAKE, FAKE, None, None) == bd.RR_ERR_PARAM
    # an fp32 block of 128 x 128 does not fit the generic kernel's LDS plan
    s2 = shape(d=128)
    assert bd.lib.rr_dense_attn(C.byref(s2), FAKE, FAKE, FAKE, 128, FAKE, None, None) == bd.RR_ERR_SHAPE


def test_binding_refuses_wrong_dtype_without_gpu():
    import torch
    q = torch.zeros((1, 2, 64, 64), dtype=torch.float16)
    with pytest.raises(bd.RRError):
        bd.make_shape(q, q)


def test_packed_sequence_argument_errors_and_table_helper():
    s = shape()
    assert bd.lib.rr_dense_attn_packed(C.byref(s), FAKE, FAKE, FAKE, 64, None, FAKE, None, None) == bd.RR_ERR_NULL
    assert bd.lib.rr_dense_attn_packed(C.byref(s), FAKE, None, FAKE, 64, FAKE, FAKE, None, None) == bd.RR_ERR_NULL
    assert bd.lib.rr_dense_attn_packed(C.byref(s), FAKE, FAKE, FAKE, 136, FAKE, FAKE, None, None) == bd.RR_ERR_SHAPE
    s.Lq = 256                                                       # a query chunk and a table do not combine
    assert bd.lib.rr_dense_attn_packed(C.byref(s), FAKE, FAKE, FAKE, 64, FAKE, FAKE, None, None) == bd.RR_ERR_PARAM
    m = bd.rr_mask(None, FAKE, FAKE, None, 16, 64, None)
    opts = bd.rr_estimate_opts(1, 0, 0, 0, 0, FAKE)
    assert bd.lib.rr_estimate_ex(C.byref(s), FAKE, FAKE, 8, 64, 0.9, C.byref(opts), FAKE * 16, 1 << 30, C.byref(m),
                                 None) == bd.RR_ERR_PARAM
    # both flag bits are known, the next one is not
    s.Lq = 0
    assert call_estimate(s, flags=3, ws=None) == bd.RR_ERR_WORKSPACE and call_estimate(s, flags=7, ws=None) == bd.RR_ERR_PARAM
    # the table of the header for sequences of 3, 1 and 4 blocks
    assert bd.packed_seq_first([3, 1, 4], "cpu").tolist() == [0, 0, 0, 3, 4, 4, 4, 4]


def test_attention_workspace_sizes_over_random_geometries():
    """Host-side planning of the calls with a workspace over seeded random shapes: sizes are multiples of 256 bytes,
    zero for a whole prefill and for shapes the matrix kernel does not serve, never smaller than one fp32 output row
    plus its lse per query row where the call is split, and a workspace 256 bytes short, or misaligned, is refused before any
    launch."""
    import random
    rnd = random.Random(2602)
    FAKE = 1 << 20
    seen = {"zero": 0, "decode": 0, "parts": 0, "plan": 0}
    for _ in range(400):
        Hkv = rnd.choice([1, 2, 4, 8])
        Hq = Hkv * rnd.choice([1, 2, 4, 7, 8])
        L = rnd.choice([777, 4096, 20000, 32768, 131072, 1 << 20]) - rnd.choice([0, 0, 59])
        Lq = rnd.choice([0, 1, 2, 3, 16, 100, 128, 129, 1000, 2048, 8192])
        if Lq > L:
            continue
        batch = rnd.choice([1, 1, 2, 3])
        s = shape(L=L, Hq=Hq, Hkv=Hkv, d=128, dtype=bd.RR_BF16, batch=batch)
        s.Lq = Lq
        need = bd.lib.rr_attn_workspace_bytes(C.byref(s), 128)
        assert need % 256 == 0
        if Lq == 0:
            assert need == 0
        if need == 0:
            seen["zero"] += 1
            continue
        rows = batch * Hq * Lq
        assert need >= rows * (128 * 4 + 4)
        seen["decode" if Lq <= 2 and (Hq // Hkv) * Lq <= 8 else ("plan" if Lq > 128 else "parts")] += 1
        assert bd.lib.rr_dense_attn_ws(C.byref(s), FAKE, FAKE, FAKE, 128, FAKE, None, FAKE, need - 256, None) == bd.RR_ERR_WORKSPACE
        assert bd.lib.rr_dense_attn_ws(C.byref(s), FAKE, FAKE, FAKE, 128, FAKE, None, FAKE + 8, need, None) == bd.RR_ERR_WORKSPACE
        s32 = shape(L=L, Hq=Hq, Hkv=Hkv, d=64, dtype=bd.RR_F32, batch=batch)
        s32.Lq = Lq
        assert bd.lib.rr_attn_workspace_bytes(C.byref(s32), 64) == 0
    assert min(seen.values()) > 5, seen
