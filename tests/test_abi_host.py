"""Host-only checks of the C ABI: the library loads without a GPU, exports every
symbol the header declares, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

import oracle
from paper_2406_11430_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "l2kv.h")

OK, E_NULL, E_SHAPE, E_DTYPE, E_RATIO, E_WS, E_ALIGN, E_LAUNCH = 0, -1, -2, -3, -4, -5, -6, -7


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libl2kv.so not built: run `python -m paper_2406_11430_amd.build`")
    return binding.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(l2kv_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported_and_bound(lib):
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), "symbol %s missing from libl2kv.so" % n
        assert n in binding.SIGNATURES, "no ctypes signature for %s" % n
    for n in binding.SIGNATURES:
        assert n in names, "binding declares %s which the header does not" % n


def test_python_binding_has_same_names():
    import paper_2406_11430_amd as pkg
    for n in declared_functions():
        if n in ("l2kv_status_string",):
            continue
        assert callable(getattr(pkg, n, None)), "python binding lacks %s" % n


def test_status_strings(lib):
    seen = set()
    for s in range(0, -8, -1):
        txt = lib.l2kv_status_string(s).decode()
        assert txt and txt != "unknown status"
        seen.add(txt)
    assert len(seen) == 8
    assert lib.l2kv_status_string(-99).decode() == "unknown status"


@pytest.mark.parametrize("T,r", [(512, 0.5), (4096, 0.5), (131072, 0.1), (100, 0.55), (100, 0.07),
                                 (10, 0.3), (7, 0.5), (8, 0.3), (8, 1.0), (1, 0.01), (1000, 1e-9),
                                 (3, 0.999), (12345, 0.3333), (99999, 0.9)])
def test_keep_count_agrees_with_oracle(lib, T, r):
    assert lib.l2kv_keep_count(T, r) == oracle.keep_count(T, r)


def test_keep_count_rejects_bad_ratio(lib):
    for r in (0.0, -0.5, 1.0000001, float("nan"), float("inf")):
        assert lib.l2kv_keep_count(100, r) == 0
    assert lib.l2kv_keep_count(0, 0.5) == 0 and lib.l2kv_keep_count(-3, 0.5) == 0


P = 0x1000   # a non-null, 16-aligned fake device address: never dereferenced on these paths


def test_norms_validation(lib):
    f = lib.l2kv_norms
    assert f(None, 1, 1, 8, 128, 1024, P, None) == E_NULL
    assert f(P, 1, 1, 8, 128, 1024, None, None) == E_NULL
    assert f(P, 7, 1, 8, 128, 1024, P, None) == E_DTYPE
    assert f(P, 1, 0, 8, 128, 1024, P, None) == E_SHAPE
    assert f(P, 1, 1, 0, 128, 1024, P, None) == E_SHAPE
    assert f(P, 1, 1, 8, 96, 1024, P, None) == E_SHAPE          # unsupported D
    assert f(P, 1, 1, 8, 128, 1023, P, None) == E_SHAPE         # stride < T*D
    assert f(P, 1, 1, 2 ** 31, 128, 2 ** 40, P, None) == E_SHAPE
    assert f(P + 8, 1, 1, 8, 128, 1024, P, None) == E_ALIGN
    assert f(P, 1, 1, 8, 128, 1024, P + 2, None) == E_ALIGN
    assert f(P, 1, 2, 8, 64, 515, P, None) == E_ALIGN           # 515*2 bytes not /16


def test_select_validation(lib):
    f = lib.l2kv_select
    ws = lib.l2kv_select_workspace_bytes(4, 100)
    assert ws > 0
    assert f(None, 4, 100, 0.5, P, None, P, ws, None) == E_NULL
    assert f(P, 4, 100, 0.5, None, None, P, ws, None) == E_NULL
    assert f(P, 0, 100, 0.5, P, None, P, ws, None) == E_SHAPE
    assert f(P, 4, 0, 0.5, P, None, P, ws, None) == E_SHAPE
    for r in (0.0, -1.0, 1.5, float("nan")):
        assert f(P, 4, 100, r, P, None, P, ws, None) == E_RATIO
    assert f(P, 4, 100, 0.5, P, None, None, ws, None) == E_WS
    assert f(P, 4, 100, 0.5, P, None, P, ws - 1, None) == E_WS
    assert f(P, 4, 100, 0.5, P + 2, None, P, ws, None) == E_ALIGN
    assert f(P, 4, 100, 0.5, P, None, P + 4, ws, None) == E_ALIGN
    g = lib.l2kv_select_k
    assert g(P, 4, 100, 0, 0, P, None, P, ws, None) == E_SHAPE
    assert g(P, 4, 100, 101, 0, P, None, P, ws, None) == E_SHAPE
    assert g(P, 4, 100, 10, 5, P, None, P, ws, None) == E_SHAPE   # bad mode


def test_compact_validation(lib):
    f = lib.l2kv_compact
    assert f(None, P, 1, P, 1, 8, 4, 128, 1024, P, P, None) == E_NULL
    assert f(P, P, 1, None, 1, 8, 4, 128, 1024, P, P, None) == E_NULL
    assert f(P, P, 1, P, 1, 8, 4, 128, 1024, None, P, None) == E_NULL
    assert f(P, None, 1, P, 1, 8, 4, 128, 1024, P, P, None) == E_NULL   # V without Vc
    assert f(P, P, 1, P, 1, 8, 4, 128, 1024, P, None, None) == E_NULL
    assert f(P, P, 3, P, 1, 8, 4, 128, 1024, P, P, None) == E_DTYPE
    assert f(P, P, 1, P, 1, 8, 0, 128, 1024, P, P, None) == E_SHAPE
    assert f(P, P, 1, P, 1, 8, 9, 128, 1024, P, P, None) == E_SHAPE     # k > T
    assert f(P, P, 1, P, 1, 8, 4, 32, 1024, P, P, None) == E_SHAPE
    assert f(P, P + 4, 1, P, 1, 8, 4, 128, 1024, P, P, None) == E_ALIGN
    assert f(P, P, 1, P, 1, 8, 4, 128, 1024, P, P + 8, None) == E_ALIGN


def test_compress_validation(lib):
    f = lib.l2kv_compress
    ok = [P, P, 1, 4, 1000, 128, 128000, 0.5, 0, P, P, P, P, P, 256, None]
    names = ["K", "V", "dt", "n_heads", "T", "D", "stride", "ratio", "slab", "norms", "idx", "Kc", "Vc", "ws",
             "ws_bytes", "stream"]

    def call(**kw):
        args = list(ok)
        for key, val in kw.items():
            args[names.index(key)] = val
        return f(*args)

    for key in ("K", "V", "norms", "idx", "Kc", "Vc"):
        assert call(**{key: None}) == E_NULL
    assert call(dt=3) == E_DTYPE
    assert call(n_heads=0) == E_SHAPE and call(T=0) == E_SHAPE and call(D=96) == E_SHAPE
    assert call(stride=127999) == E_SHAPE and call(slab=-1) == E_SHAPE
    assert call(ratio=0.0) == E_RATIO and call(ratio=1.5) == E_RATIO and call(ratio=float("nan")) == E_RATIO
    assert call(ws=None) == E_WS and call(ws_bytes=8) == E_WS
    assert call(K=P + 2) == E_ALIGN and call(Vc=P + 8) == E_ALIGN and call(ws=P + 4) == E_ALIGN


def test_decode_validation(lib):
    f = lib.l2kv_decode_attn
    ws = lib.l2kv_decode_workspace_bytes(2, 8, 100, 128)
    assert ws == (256 + 2 * 8 * lib.l2kv_decode_max_splits(100) * 132 * 4 + 255) // 256 * 256   # counters + partials, padded
    a = (P, P, P, 1, 2, 8, 2, 100, 128, 12800, 0.0, P, P, ws, None)

    def call(**kw):
        names = ["Q", "Kc", "Vc", "dt", "B", "Hq", "Hkv", "kv_len", "D", "stride", "scale", "O", "ws",
                 "ws_bytes", "stream"]
        args = list(a)
        for key, val in kw.items():
            args[names.index(key)] = val
        return f(*args)

    for key in ("Q", "Kc", "Vc", "O"):
        assert call(**{key: None}) == E_NULL
    assert call(dt=2) == E_DTYPE
    assert call(B=0) == E_SHAPE and call(Hq=0) == E_SHAPE and call(kv_len=0) == E_SHAPE
    assert call(Hq=7) == E_SHAPE              # not a multiple of Hkv
    assert call(Hq=18) == E_SHAPE             # group of 9 > 8
    assert call(D=80) == E_SHAPE
    assert call(D=256, stride=25600, dt=0) == E_SHAPE                 # rows of 256 elements: bf16 only,
    assert call(D=256, stride=25600, Hq=10) == E_SHAPE                # and groups of at most 4 query heads
    assert call(stride=100 * 128 - 1) == E_SHAPE
    assert call(scale=float("nan")) == E_SHAPE
    assert call(ws=None) == E_WS and call(ws_bytes=ws - 1) == E_WS
    assert call(Q=P + 4) == E_ALIGN and call(O=P + 1) == E_ALIGN and call(ws=P + 8) == E_ALIGN
    g = lib.l2kv_decode_attn_splits
    assert g(P, P, P, 1, 2, 8, 2, 100, 128, 12800, 0.0, 3, P, P, ws, None) == E_SHAPE   # > max splits (2)
    assert g(P, P, P, 1, 2, 8, 2, 100, 128, 12800, 0.0, -1, P, P, ws, None) == E_SHAPE


def test_decode_out_validation(lib):
    f = lib.l2kv_decode_attn_out
    ws = lib.l2kv_decode_workspace_bytes(2, 8, 100, 128)
    ok = (P, P, P, 1, 2, 8, 2, 100, 128, 12800, 0.0, 1, P, P, ws, None)
    names = ["Q", "Kc", "Vc", "dt", "B", "Hq", "Hkv", "kv_len", "D", "stride", "scale", "out_dt", "O", "ws",
             "ws_bytes", "stream"]

    def call(**kw):
        args = list(ok)
        for key, val in kw.items():
            args[names.index(key)] = val
        return f(*args)

    for key in ("Q", "Kc", "Vc", "O"):
        assert call(**{key: None}) == E_NULL
    assert call(out_dt=7) == E_DTYPE and call(dt=9) == E_DTYPE
    assert call(Hq=18) == E_SHAPE and call(kv_len=-1) == E_SHAPE
    assert call(ws=None) == E_WS and call(ws_bytes=ws - 16) == E_WS
    assert call(O=P + 2, out_dt=0) == E_ALIGN          # fp32 output needs 4-byte alignment
    assert call(O=P + 1) == E_ALIGN                     # bf16 output needs 2
    assert call(Q=P + 8) == E_ALIGN


def test_decode_static_validation(lib):
    f = lib.l2kv_decode_attn_static
    ok = (P, P, P, 1, 2, 8, 2, 100, 128, 12800, 0.0, P, None)
    names = ["Q", "Kc", "Vc", "dt", "B", "Hq", "Hkv", "kv_len", "D", "stride", "scale", "O", "stream"]

    def call(**kw):
        args = list(ok)
        for key, val in kw.items():
            args[names.index(key)] = val
        return f(*args)

    for key in ("Q", "Kc", "Vc", "O"):
        assert call(**{key: None}) == E_NULL
    assert call(dt=5) == E_DTYPE
    assert call(B=0) == E_SHAPE and call(Hq=18) == E_SHAPE and call(D=80) == E_SHAPE and call(kv_len=0) == E_SHAPE
    assert call(stride=100 * 128 - 1) == E_SHAPE and call(scale=float("inf")) == E_SHAPE
    assert call(Q=P + 4) == E_ALIGN and call(O=P + 2) == E_ALIGN
    # beyond the scratch array: 4096 sequences x 8 heads x 132 floats of partials alone exceed 4 MiB
    assert call(B=4096, Hq=8, Hkv=8, kv_len=64, stride=64 * 128) == E_WS
    header = open(HEADER).read()
    assert re.search(r"#define\s+L2KV_STATIC_SCRATCH_BYTES\s+\(4u << 20\)", header)


def test_workspace_init_and_random_keys_validation(lib):
    f = lib.l2kv_decode_workspace_init
    assert f(None, 256, None) == E_NULL
    assert f(P, 0, None) == E_WS and f(P, 100, None) == E_WS      # not a multiple of 16
    assert f(P + 8, 256, None) == E_ALIGN
    g = lib.l2kv_random_keys
    assert g(4, 100, 1, None, None) == E_NULL
    assert g(0, 100, 1, P, None) == E_SHAPE and g(4, 0, 1, P, None) == E_SHAPE
    assert g(4, 100, 1, P + 2, None) == E_ALIGN
    for B, Hq, n, D in ((1, 1, 1, 64), (4, 32, 16384, 128), (3, 7, 1000, 128)):
        assert lib.l2kv_decode_workspace_bytes(B, Hq, n, D) % 16 == 0


def test_read_probe_validation(lib):
    f = lib.l2kv_read_probe
    assert f(None, 1 << 20, P, None) == E_NULL
    assert f(P, 1 << 20, None, None) == E_NULL
    assert f(P + 8, 1 << 20, P, None) == E_ALIGN
    assert f(P, 1 << 20, P + 2, None) == E_ALIGN
    assert f(P, 8191, P, None) == E_SHAPE            # less than one block of 8192 bytes
    assert f(P, 8192 << 31, P, None) == E_SHAPE      # more blocks than a grid holds


def test_decode_max_splits(lib):
    assert lib.l2kv_decode_max_splits(0) == 0
    assert lib.l2kv_decode_max_splits(1) == 1
    assert lib.l2kv_decode_max_splits(64) == 1
    assert lib.l2kv_decode_max_splits(65) == 2
    assert lib.l2kv_decode_max_splits(16384) == 256
    assert lib.l2kv_decode_max_splits(10 ** 6) == 256


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2406_11430_amd as pkg
    K = torch.zeros(1, 8, 128, dtype=torch.bfloat16)
    n = torch.zeros(1, 8)
    with pytest.raises(ValueError):
        pkg.l2kv_norms(K, n)


def test_ragged_and_stream_validation(lib):
    sel = lib.l2kv_select_ragged
    assert sel(None, 8, 4, 1000, P, P, 500, 300, 0, P, None) == E_NULL
    assert sel(P, 8, 4, 1000, None, P, 500, 300, 0, P, None) == E_NULL
    assert sel(P, 0, 4, 1000, P, P, 500, 300, 0, P, None) == E_SHAPE
    assert sel(P, 8, 4, 1000, P, P, 1001, 300, 0, P, None) == E_SHAPE      # kept > tokens
    assert sel(P, 8, 4, 1000, P, P, 500, 0, 0, P, None) == E_SHAPE
    assert sel(P, 8, 4, 1000, P, P, 500, 300, 7, P, None) == E_SHAPE       # bad mode
    assert sel(P, 8, 4, 1000, P + 4, P, 500, 300, 0, P, None) == E_ALIGN   # int64 offsets need 8
    cmp_ = lib.l2kv_compact_ragged
    ok = [P, P, P, 1, P, 8, 4, 1000, P, P, 500, 200, P, 600, 128, P, P, P, P, None]
    for i in (0, 1, 2, 4, 8, 9, 12, 15, 16, 17, 18):
        bad = list(ok)
        bad[i] = None
        assert cmp_(*bad) == E_NULL, i
    bad = list(ok); bad[3] = 9
    assert cmp_(*bad) == E_DTYPE
    bad = list(ok); bad[14] = 100
    assert cmp_(*bad) == E_SHAPE
    bad = list(ok); bad[11] = 501                                         # max_kept > total_kept
    assert cmp_(*bad) == E_SHAPE
    bad = list(ok); bad[15] = P + 8
    assert cmp_(*bad) == E_ALIGN
    app = lib.l2kv_stream_append
    ok = [P, P, 1, 2, 4, 8, 128, P, P, 600, P, P + 64, P, P, P, P, None]
    assert app(*[None] + ok[1:]) == E_NULL
    bad = list(ok); bad[11] = bad[10]
    assert app(*bad) == E_SHAPE                                           # lens_out aliases lens_in
    bad = list(ok); bad[6] = 48
    assert app(*bad) == E_SHAPE
    bad = list(ok); bad[8] = P + 4
    assert app(*bad) == E_ALIGN
    ev = lib.l2kv_stream_evict
    ok = [1, 16, 4, 128, P, 600, P, P, P + 64, P, P, P, P, None]
    bad = list(ok); bad[7] = None
    assert ev(*bad) == E_NULL
    bad = list(ok); bad[8] = bad[6]
    assert ev(*bad) == E_SHAPE
    bad = list(ok); bad[0] = 5
    assert ev(*bad) == E_DTYPE
    dec = lib.l2kv_decode_attn_ragged
    ws = lib.l2kv_decode_ragged_workspace_bytes(4, 8, 300, 128)
    assert ws == lib.l2kv_decode_workspace_bytes(4, 8, 300, 128) + 256     # + room for a launch order
    # Q Kc Vc dt n_seq Hq Hkv D lens slot_off seq_order total_slots max_len scale n_splits O ws ws_bytes stream
    ok = [P, P, P, 1, 4, 8, 2, 128, P, P, None, 600, 300, 0.0, 0, P, P, ws, None]
    assert dec(*ok[:8] + [None] + ok[9:]) == E_NULL
    bad = list(ok); bad[12] = 601                                         # max_len > total_slots
    assert dec(*bad) == E_SHAPE
    bad = list(ok); bad[14] = 99
    assert dec(*bad) == E_SHAPE
    bad = list(ok); bad[17] = ws - 1
    assert dec(*bad) == E_WS
    bad = list(ok); bad[9] = P + 4
    assert dec(*bad) == E_ALIGN
    bad = list(ok); bad[10] = P + 2                                       # seq_order given but misaligned
    assert dec(*bad) == E_ALIGN
    order = lib.l2kv_length_order
    assert order(None, 4, P, None) == E_NULL and order(P, 4, None, None) == E_NULL
    assert order(P, 0, P + 64, None) == E_SHAPE and order(P, 70000, P + 64, None) == E_SHAPE
    assert order(P, 4, P, None) == E_SHAPE                                # in place
    assert order(P + 2, 4, P + 64, None) == E_ALIGN


def test_attention_loss_validation(lib):
    wr = lib.l2kv_norm_ranks_workspace_bytes(3, 1000)
    assert wr == (3 * 1000 * 16 + 255) // 256 * 256 and lib.l2kv_norm_ranks_workspace_bytes(0, 5) == 0
    f = lib.l2kv_norm_ranks
    assert f(None, 3, 1000, P, P, wr, None) == E_NULL and f(P, 3, 1000, None, P, wr, None) == E_NULL
    assert f(P, 0, 1000, P, P, wr, None) == E_SHAPE and f(P, 3, 0, P, P, wr, None) == E_SHAPE
    assert f(P, 3, 2 ** 31, P, P, wr, None) == E_SHAPE
    assert f(P, 3, 1000, P, None, wr, None) == E_WS and f(P, 3, 1000, P, P, wr - 1, None) == E_WS
    assert f(P + 2, 3, 1000, P, P, wr, None) == E_ALIGN and f(P, 3, 1000, P, P + 8, wr, None) == E_ALIGN

    wa = lib.l2kv_alr_workspace_bytes(2, 8, 100)
    assert wa == (2 * 8 * 100 * 8 + 255) // 256 * 256 and lib.l2kv_alr_workspace_bytes(2, 8, 0) == 0
    g = lib.l2kv_alr
    a = (P, P, 1, P, 2, 8, 2, 100, 128, 12800, 0.0, 50, P, P, P, P, wa, None)
    names = ["Q", "K", "dt", "rank", "B", "Hq", "Hkv", "T", "D", "stride", "scale", "m", "alr", "loss",
             "loss_ref", "ws", "ws_bytes", "stream"]

    def call(**kw):
        args = list(a)
        for key, val in kw.items():
            args[names.index(key)] = val
        return g(*args)

    for key in ("Q", "K", "rank", "alr"):
        assert call(**{key: None}) == E_NULL
    assert call(dt=5) == E_DTYPE
    assert call(B=0) == E_SHAPE and call(T=0) == E_SHAPE and call(D=96) == E_SHAPE
    assert call(Hq=7) == E_SHAPE and call(Hq=18) == E_SHAPE
    assert call(stride=100 * 128 - 1) == E_SHAPE
    assert call(m=-1) == E_SHAPE and call(m=101) == E_SHAPE
    assert call(scale=float("inf")) == E_SHAPE
    assert call(ws=None) == E_WS and call(ws_bytes=wa - 1) == E_WS
    assert call(Q=P + 4) == E_ALIGN and call(alr=P + 4) == E_ALIGN and call(loss=P + 4) == E_ALIGN
    assert call(ws=P + 8) == E_ALIGN


def test_header_is_plain_c_and_cpp(tmp_path):
    # the boundary is a C ABI: the header must compile on its own as C99 and as C++
    import subprocess
    src_c = tmp_path / "use_header.c"
    src_c.write_text('#include "l2kv.h"\nint main(void) { return (int)l2kv_keep_count(8, 0.5) == 4 ? 0 : 1; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(src_c)],
                   check=True)
    src_cpp = tmp_path / "use_header.cpp"
    src_cpp.write_text('#include "l2kv.h"\nint main() { return l2kv_version() > 0 ? 0 : 1; }\n')
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(src_cpp)], check=True)
    # and a C program links against the library and runs its host-only entry points
    exe = tmp_path / "use_header"
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src_c), "-o", str(exe), binding.LIB_PATH,
                    "-Wl,-rpath," + os.path.dirname(binding.LIB_PATH)], check=True)
    assert subprocess.run([str(exe)]).returncode == 0
