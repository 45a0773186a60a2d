"""The allocation-free decode entry point (l2kv_decode_attn_static), called
through the C ABI with raw device addresses, against l2kv_decode_attn with a
caller-provided workspace: two calls in a row on the same GPU, the second on a
smaller input, so the second call runs over what the first left in the
library's scratch array.  Both entry points launch the same kernels with the
same decomposition, so the outputs must be bit-identical; they are also held to
the attention tolerance against the CPU oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import paper_2406_11430_amd as l2kv
from paper_2406_11430_amd import binding, synth

pytestmark = pytest.mark.gpu

ATTN_GATE = 2e-3
ATTN_BAR = 1e-4
SCRATCH_BYTES = 4 << 20     # L2KV_STATIC_SCRATCH_BYTES of include/l2kv.h


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.fail("no HIP device visible: the gpu tests need a real MI355X")
    l2kv.lib()
    return torch.device("cuda:0")


def make_case(seed, B, Hkv, G, n, D, dev):
    rng = np.random.default_rng(seed)
    bf = lambda a: torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)     # noqa: E731
    K = bf(rng.standard_normal((B, Hkv, n, D)) * np.exp(0.5 * rng.standard_normal((B, Hkv, n, 1))))
    V = bf(rng.standard_normal((B, Hkv, n, D)))
    Q = bf(rng.standard_normal((B, Hkv * G, D)))
    return (Q, K, V), tuple(t.to(dev) for t in (Q, K, V))


def raw_static(Qd, Kd, Vd):
    """The new entry point through ctypes with plain addresses and sizes."""
    B, Hq, D = Qd.shape
    _, Hkv, n, _ = Kd.shape
    O = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device=Qd.device)
    st = binding.lib().l2kv_decode_attn_static(
        C.c_void_p(Qd.data_ptr()), C.c_void_p(Kd.data_ptr()), C.c_void_p(Vd.data_ptr()), binding.L2KV_BF16,
        B, Hq, Hkv, n, D, n * D, 0.0, C.c_void_p(O.data_ptr()),
        C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, binding.lib().l2kv_status_string(st).decode()
    return O


def raw_workspace(Qd, Kd, Vd):
    """The existing entry point, same way, with a fresh zeroed workspace."""
    B, Hq, D = Qd.shape
    _, Hkv, n, _ = Kd.shape
    lib = binding.lib()
    nbytes = lib.l2kv_decode_workspace_bytes(B, Hq, n, D)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=Qd.device)
    O = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device=Qd.device)
    st = lib.l2kv_decode_attn(
        C.c_void_p(Qd.data_ptr()), C.c_void_p(Kd.data_ptr()), C.c_void_p(Vd.data_ptr()), binding.L2KV_BF16,
        B, Hq, Hkv, n, D, n * D, 0.0, C.c_void_p(O.data_ptr()), C.c_void_p(ws.data_ptr()), nbytes,
        C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0
    return O


def test_static_scratch_decode_two_calls_second_smaller(dev):
    # first call: 3 sequences x 2 KV heads x 4 query heads each, 5003 rows (several workgroups per
    # head and a ragged last tile); second call: fewer sequences, heads and rows
    shapes = [(11, 3, 2, 4, 5003, 128), (12, 1, 2, 2, 777, 128)]
    cases = [make_case(*s, dev) for s in shapes]
    got = []
    for _, (Qd, Kd, Vd) in cases:                 # the two static calls back to back, nothing in between
        got.append(raw_static(Qd, Kd, Vd))
    torch.cuda.synchronize()
    for (host, (Qd, Kd, Vd)), O_static in zip(cases, got):
        O_ws = raw_workspace(Qd, Kd, Vd)
        torch.cuda.synchronize()
        assert torch.equal(O_static, O_ws), "static-scratch result differs from the workspace entry point"
        Q, K, V = (synth.as_numpy_bits(t) for t in host)
        want = oracle.decode_attn(Q, K, V, "bf16")
        err = float(np.abs(O_static.cpu().numpy() - want).max())
        assert err <= ATTN_BAR and err <= ATTN_GATE, err


def test_static_scratch_repeats_and_rejects_oversize(dev):
    (_, (Qd, Kd, Vd)) = make_case(13, 2, 2, 4, 4096, 128, dev)
    first = raw_static(Qd, Kd, Vd)
    again = raw_static(Qd, Kd, Vd)
    torch.cuda.synchronize()
    assert torch.equal(first, again)
    # a shape whose partials cannot fit the scratch array is refused on the host, nothing is
    # launched: 4096 sequences x 8 query heads x 132 floats > 4 MiB (addresses are never read)
    lib = binding.lib()
    P = C.c_void_p(0x1000)
    st = lib.l2kv_decode_attn_static(P, P, P, binding.L2KV_BF16, 4096, 8, 8, 64, 128, 64 * 128, 0.0, P, None)
    assert st == -5
    assert 256 * 64 + 4096 * 8 * 132 * 4 > SCRATCH_BYTES
