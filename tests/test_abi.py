"""Host-side checks of the C ABI: the library loads, exports every symbol the
header declares, classifies steps like the oracle, and rejects bad arguments
before launching anything (fake non-null pointers; no GPU needed)."""
import ctypes
import os
import re

import pytest

from oracle import striped_attention as orc
from paper_2311_09431_amd import binding as sa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "striped_attn.h")) as f:
        text = f.read()
    declared = set(re.findall(r"\b(sa_[a-z_]+)\s*\(", text))
    assert declared == set(sa.EXPORTS)
    L = sa.lib()
    for name in declared:
        assert getattr(L, name) is not None


@pytest.mark.parametrize("N,c", [(4, 4), (8, 3), (1, 5)])
def test_step_mask_and_pairs_match_the_oracle(N, c):
    import numpy as np
    for layout in (sa.CONTIGUOUS, sa.STRIPED):
        for j in range(N):
            for k in range(N):
                kind, off = sa.sa_step_mask(j, k, N, layout)
                allowed = orc.get_mask(j, k, N, c, layout)
                a = np.arange(c)[:, None]
                b = np.arange(c)[None, :]
                if kind == sa.MASK_EMPTY:
                    mine = np.zeros((c, c), bool)
                elif kind == sa.MASK_FULL:
                    mine = np.ones((c, c), bool)
                else:
                    mine = b <= a - off
                assert (mine == allowed).all()
                assert sa.sa_step_pairs(j, k, N, layout, c) == orc.work(j, k, N, c, layout)


def _shape(**kw):
    base = dict(B=1, H=2, c=64, d=64, stride_b=2 * 256 * 64, stride_h=256 * 64, stride_s=0, stat_stride_b=512,
                stat_stride_h=256, dtype=sa.F32, softmax_scale=0.0)
    base.update(kw)
    return sa.SaShape(**base)


def test_argument_errors_are_reported_before_any_launch():
    L = sa.lib()
    p = ctypes.c_void_p(0x1000)      # non-null, 16-byte aligned, never dereferenced on error paths
    odd = ctypes.c_void_p(0x1004)
    null = ctypes.c_void_p(0)
    ok = _shape()
    f = L.sa_attn_step_fwd
    assert f(null, p, p, p, p, 0, 0, 4, 0, ctypes.byref(ok), None) == -1
    assert f(p, p, p, p, p, 0, 0, 4, 0, None, None) == -1
    assert f(p, p, p, p, p, 4, 0, 4, 0, ctypes.byref(ok), None) == -3
    assert f(p, p, p, p, p, 0, -1, 4, 0, ctypes.byref(ok), None) == -3
    assert f(p, p, p, p, p, 0, 0, 0, 0, ctypes.byref(ok), None) == -3
    assert f(p, p, p, p, p, 0, 0, 4, 2, ctypes.byref(ok), None) == -5
    assert f(p, odd, p, p, p, 0, 0, 4, 0, ctypes.byref(ok), None) == -6
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(dtype=7)), None) == -4
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(d=0)), None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(d=512)), None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(d=66)), None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(c=0)), None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(stride_h=10)), None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(dtype=sa.BF16, stride_h=256 * 64 + 2)),
             None) == -6
    # fewer key/value heads: H_kv must divide H, and K/V strides obey the same rules as Q's
    kv = dict(kv_stride_b=256 * 64, kv_stride_h=256 * 64, kv_stride_s=0)
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(H=3, stride_b=3 * 256 * 64, H_kv=2, **kv)), None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(H_kv=-1, **kv)), None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(H_kv=1, kv_stride_b=0, kv_stride_h=8, kv_stride_s=0)),
             None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(H_kv=1, kv_stride_b=0, kv_stride_h=64 * 64,
                                                           kv_stride_s=32)), None) == -2
    assert f(p, p, p, p, p, 0, 0, 4, 0, ctypes.byref(_shape(H_kv=1, kv_stride_b=0, kv_stride_h=64 * 66,
                                                           kv_stride_s=66)), None) == -6
    # with H_kv = 0 the K/V fields are not looked at
    assert f(p, p, p, p, p, 0, 1, 4, sa.CONTIGUOUS, ctypes.byref(_shape(H_kv=0, kv_stride_h=-5)), None) == 0
    # an entirely masked contiguous step is a no-op that succeeds without a launch
    assert f(p, p, p, p, p, 0, 1, 4, sa.CONTIGUOUS, ctypes.byref(ok), None) == 0

    # forward step with the fused query rotation: its own arguments, and only shapes the
    # matrix-core forward kernel takes (bf16, d = 64 / 128 / 256, c a multiple of 128)
    fr = L.sa_attn_step_fwd_rope
    big = dict(dtype=sa.BF16, c=256, d=128, stride_b=2 * 1024 * 128, stride_h=1024 * 128, stat_stride_b=2048,
               stat_stride_h=1024)
    good = _shape(**big)
    assert fr(p, p, p, p, p, null, 0, 10000.0, 0, 0, 4, 0, ctypes.byref(good), None) == -1
    assert fr(p, p, p, p, p, ctypes.c_void_p(0x1002), 0, 10000.0, 0, 1, 4, 0, ctypes.byref(good), None) == -6
    assert fr(p, p, p, p, p, p, 0, 1.0, 0, 1, 4, 0, ctypes.byref(good), None) == -2          # base must exceed 1
    assert fr(p, p, p, p, p, p, 100, 10000.0, 0, 1, 4, 0, ctypes.byref(good), None) == -2      # id rows overlap
    assert fr(p, p, p, p, p, p, 0, 10000.0, 0, 1, 4, 0, ctypes.byref(ok), None) == -2         # fp32: generic kernels
    assert fr(p, p, p, p, p, p, 0, 10000.0, 0, 1, 4, 0, ctypes.byref(_shape(**dict(big, d=100, stride_h=1024 * 100,
              stride_b=2 * 1024 * 100))), None) == -2
    assert fr(p, p, p, p, p, p, 0, 10000.0, 0, 1, 4, 0, ctypes.byref(_shape(**dict(big, c=192))), None) == -2
    assert fr(p, p, p, p, p, p, 0, 10000.0, 5, 1, 4, 0, ctypes.byref(good), None) == -3
    # an entirely masked step with valid arguments: success, nothing launched
    assert fr(p, p, p, p, p, p, 0, 10000.0, 0, 1, 4, sa.CONTIGUOUS, ctypes.byref(good), None) == 0

    g = L.sa_stripe_permute
    assert g(null, p, 1, 16, 4, 4, None) == -1
    assert g(p, p, 1, 16, 4, 4, None) == -5
    assert g(p, odd, 1, 16, 8, 4, None) == -6
    assert g(p, ctypes.c_void_p(0x2000), 1, 18, 4, 4, None) == -2
    assert g(p, ctypes.c_void_p(0x2000), 1, 16, 0, 4, None) == -2
    assert g(p, ctypes.c_void_p(0x2000), 1, 16, 4, 0, None) == -3
    assert L.sa_unstripe_permute(p, ctypes.c_void_p(0x2000), 1, 18, 4, 4, None) == -2

    b = L.sa_attn_step_bwd
    assert b(p, p, p, p, p, p, p, p, null, 0, 0, 4, 0, ctypes.byref(ok), None) == -1
    assert b(p, p, p, p, p, p, p, p, p, 0, 9, 4, 0, ctypes.byref(ok), None) == -3

    r = L.sa_ring_fwd
    assert r(p, p, p, p, p, 4, 1, ctypes.byref(ok), 4, None, None) == -3
    assert r(p, p, p, p, p, 8, 1, ctypes.byref(ok), -1, None, None) == -2   # strides hold only 4 shards
    assert r(p, p, p, p, p, 4, 1, ctypes.byref(_shape(H_kv=1, kv_stride_b=0, kv_stride_h=128 * 64)), -1, None,
             None) == -2                                                    # K/V strides hold only 2 shards
    assert L.sa_state_init(p, null, ctypes.byref(ok), None) == -1
    assert L.sa_finalize(p, odd, ctypes.byref(ok), None) == -6
    assert L.sa_bwd_preprocess(p, p, null, ctypes.byref(ok), None) == -1


def test_status_strings():
    assert sa.sa_status_str(0) == "ok"
    assert "shape" in sa.sa_status_str(-2)
    assert sa.sa_status_str(-99) == "unknown status"
    assert sa.sa_step_pairs(0, 9, 4, 0, 8) == -1


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 1, 8, 4)
    with pytest.raises(TypeError):
        sa.sa_stripe_permute(x, x.clone(), 2)


def test_header_is_valid_c():
    # the boundary is a C ABI: the header must compile as plain C
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = '#include "striped_attn.h"\nint main(void) { sa_shape s; s.B = 1; return sa_status_str(SA_OK) == (const char*)0 || s.B != 1; }\n'
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", "-I",
                        os.path.join(ROOT, "include"), "-"], input=src, text=True, capture_output=True)
    assert r.returncode == 0, r.stderr


@pytest.mark.parametrize("N,c,bq,bk", [(4, 16, 4, 8), (4, 16, 8, 4), (2, 12, 3, 4), (3, 8, 8, 8), (2, 8, 1, 1)])
def test_step_tiles_match_the_oracle_classifier(N, c, bq, bk):
    for layout in (sa.CONTIGUOUS, sa.STRIPED):
        for j in range(N):
            for k in range(N):
                full, part, empty = orc.classify_tiles(orc.get_mask(j, k, N, c, layout), bq, bk)
                assert sa.sa_step_tiles(j, k, N, layout, c, bq, bk) == (full + part, full + part + empty)


def test_step_tiles_reproduce_the_printed_skipping_figures():
    # tests/golden/tiling_examples.txt: the fractions of tiles the paper says are skipped
    with open(os.path.join(ROOT, "tests", "golden", "tiling_examples.txt")) as f:
        rows = [l.split("#")[0].split() for l in f if l.split("#")[0].strip()]
    assert rows
    for c, tq, tk, mask, _full, _part, empty, pct in rows:
        c, tq, tk, empty, pct = int(c), int(tq), int(tk), int(empty), int(pct)
        # "causal" = a diagonal block (either layout with kv_dev <= q_dev); "striped_lo" = a
        # striped step with kv_dev > q_dev
        j, k = (1, 1) if mask == "causal" else (0, 1)
        computed, total = sa.sa_step_tiles(j, k, 2, sa.STRIPED, c, tq, tk)
        assert total - computed == empty
        assert round(100 * (total - computed) / total) == pct


def test_step_tiles_errors():
    L = sa.lib()
    a, b = ctypes.c_int64(), ctypes.c_int64()
    assert L.sa_step_tiles(0, 0, 2, 1, 8, 3, 4, ctypes.byref(a), ctypes.byref(b)) == -2
    assert L.sa_step_tiles(0, 0, 2, 1, 8, 0, 4, ctypes.byref(a), ctypes.byref(b)) == -2
    assert L.sa_step_tiles(0, 5, 2, 1, 8, 4, 4, ctypes.byref(a), ctypes.byref(b)) == -3
    assert L.sa_step_tiles(0, 0, 2, 7, 8, 4, 4, ctypes.byref(a), ctypes.byref(b)) == -5
    assert L.sa_step_tiles(0, 0, 2, 1, 8, 4, 4, None, ctypes.byref(b)) == -1


def test_rope_argument_errors():
    L = sa.lib()
    p = ctypes.c_void_p(0x1000)
    ok = _shape()
    f = L.sa_rope
    assert f(None, p, p, 0, ctypes.byref(ok), 10000.0, 0, None) == -1
    assert f(p, p, None, 0, ctypes.byref(ok), 10000.0, 0, None) == -1
    assert f(p, p, p, 0, ctypes.byref(ok), 1.0, 0, None) == -2          # base must exceed 1
    assert f(p, p, p, 3, ctypes.byref(ok), 10000.0, 0, None) == -2      # id rows would overlap
    assert f(p, p, ctypes.c_void_p(0x1002), 0, ctypes.byref(ok), 10000.0, 0, None) == -6
    assert f(p, p, p, 0, ctypes.byref(_shape(d=0)), 10000.0, 0, None) == -2


@pytest.mark.gpu
def test_device_props_are_those_of_an_mi355x():
    cus, khz, mem = sa.sa_device_props()
    assert cus == 256 and 1_000_000 <= khz <= 3_000_000 and mem > 200 * 2 ** 30
