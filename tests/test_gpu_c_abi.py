"""The library driven by a plain C program (tests/abi_c/l2kv_c_driver.c): hipMalloc
memory, the C ABI, no Python and no tensor library in the process that runs the
kernels.  The program writes its results to a file; this test rebuilds the same
inputs (an integer mix of the element index, no arithmetic of the method) and
checks the file against the CPU oracle: norm bits, kept indices and compacted
rows exactly, attention within the tolerance."""
import os
import subprocess

import numpy as np
import pytest

import oracle
from paper_2406_11430_amd import build

pytestmark = pytest.mark.gpu
ATTN_BAR = 1e-4


def unit_value(i, salt):
    x = (i.astype(np.uint32) * np.uint32(2654435761) + np.uint32(salt)).astype(np.uint32)
    x ^= x >> np.uint32(15); x *= np.uint32(0x2C1B3C6D); x ^= x >> np.uint32(12)
    x *= np.uint32(0x297A2D39); x ^= x >> np.uint32(15)
    return ((x >> np.uint32(9)) & np.uint32(0x3FFF)).astype(np.float32) * np.float32(1.0 / 8192.0) - np.float32(1.0)


def bf16_bits(f):
    return (f.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


@pytest.mark.parametrize("B,Hkv,G,T,r", [(2, 3, 4, 2000, 0.5), (1, 2, 1, 777, 0.1)])
def test_c_program_runs_the_hot_path(tmp_path, B, Hkv, G, T, r):
    if not os.path.exists(build.C_DRIVER_BIN):
        pytest.fail("tests/abi_c/l2kv_c_driver is not built: run `python -m paper_2406_11430_amd.build`")
    out = tmp_path / "out.bin"
    res = subprocess.run([build.C_DRIVER_BIN, str(out), str(B), str(Hkv), str(G), str(T), repr(r)],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    D, Hq, n_heads = 128, Hkv * G, B * Hkv
    k = oracle.keep_count(T, r)
    raw = out.read_bytes()
    header = np.frombuffer(raw, dtype=np.int64, count=5)
    assert list(header) == [n_heads, T, k, Hq, D]
    pos = 40

    def take(dtype, count):
        nonlocal pos
        a = np.frombuffer(raw, dtype=dtype, count=count, offset=pos)
        pos += a.nbytes
        return a

    norms = take(np.float32, n_heads * T).reshape(n_heads, T)
    idx = take(np.int32, n_heads * k).reshape(n_heads, k)
    Kc = take(np.uint16, n_heads * k * D).reshape(B, Hkv, k, D)
    Vc = take(np.uint16, n_heads * k * D).reshape(B, Hkv, k, D)
    O = take(np.float32, B * Hq * D).reshape(B, Hq, D)
    O_static = take(np.float32, B * Hq * D).reshape(B, Hq, D)
    assert pos == len(raw)

    # the same inputs, rebuilt
    i = np.arange(n_heads * T * D, dtype=np.uint32)
    scale = np.float32(0.25) + (((i // np.uint32(D)) * np.uint32(37)) % np.uint32(64)).astype(np.float32) * np.float32(1.0 / 32.0)
    K = bf16_bits(unit_value(i, 0x11) * scale).reshape(B, Hkv, T, D)
    V = bf16_bits(unit_value(i, 0x22)).reshape(B, Hkv, T, D)
    j = np.arange(B * Hq * D, dtype=np.uint32)
    Q = bf16_bits(unit_value(j, 0x33) * np.float32(4.0)).reshape(B, Hq, D)

    n32, _, want_idx, want_K, want_V = oracle.compress(K, V, "bf16", r)
    assert np.array_equal(norms.view(np.uint32), n32.reshape(n_heads, T).view(np.uint32))
    assert np.array_equal(idx, want_idx.reshape(n_heads, k))
    assert np.array_equal(Kc, want_K) and np.array_equal(Vc, want_V)
    want_O = oracle.decode_attn(Q, want_K, want_V, "bf16")
    assert np.abs(O - want_O).max() <= ATTN_BAR
    assert np.array_equal(O.view(np.uint32), O_static.view(np.uint32))
