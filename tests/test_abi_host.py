"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
include/taco.h declares, answers the size queries and rejects bad arguments before any
launch."""
import ctypes
import os
import re

import pytest

from paper_2604_24088_amd import taco

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="taco.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(taco_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = taco.lib()
    names = declared_functions()
    assert set(names) == set(taco.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None, name
    debug = declared_functions("taco_debug.h")
    assert set(debug) == set(taco.DEBUG_EXPORTS)          # the diagnostics have a header of their own
    for name in debug:
        assert getattr(L, name) is not None, name


def test_library_matches_the_sources():
    """The loaded library was built from the sources on disk (its embedded digest is theirs)."""
    from paper_2604_24088_amd import build
    assert taco.taco_build_id() == build.source_digest() == build.library_digest()
    assert not build.is_stale()


def test_version_and_strerror():
    assert re.fullmatch(r"\d+\.\d+", taco.taco_version())
    assert taco.taco_strerror(0) == "ok"
    for st in range(-13, 0):
        assert taco.taco_strerror(st) not in ("ok", "unknown status")
    assert taco.taco_strerror(-100) == "unknown status"


def test_default_params():
    p = taco.taco_default_params()
    assert (p.block, p.format, p.impl, p.layout, p.mode) == (128, 0, 0, 0, 7)
    assert p.tau == 1.0 and abs(p.eps - 1e-12) < 1e-18


@pytest.mark.parametrize("n,block,codes,scales", [
    (262144, 128, 262144, 16384), (1, 128, 128, 8), (129, 128, 256, 16), (33554432, 256, 33554432, 1048576),
    (100, 32, 128, 32), (0, 128, 0, 0), (-5, 128, 0, 0), (1000, 100, 0, 0)])
def test_size_queries(n, block, codes, scales):
    assert taco.taco_payload_bytes(n, block) == codes
    assert taco.taco_scales_bytes(n, block) == scales


def _params(**kw):
    p = taco.taco_default_params()
    for k, v in kw.items():
        setattr(p, k, v)
    return p


A = 0x1000  # a fake, 16-byte aligned, non-null "device pointer": never dereferenced on these paths


@pytest.mark.parametrize("args,status", [
    (dict(x=0), -1), (dict(payload=0), -1), (dict(scales=0), -1), (dict(p=None), -1),
    (dict(rows=0), -2), (dict(cols=-4), -2), (dict(rows=1 << 30, cols=1 << 30), -2), (dict(rows=1 << 18, cols=(1 << 18) + 1), -2),
    (dict(p=_params(block=96)), -3), (dict(p=_params(block=1024)), -3),
    (dict(x=A + 2), -4), (dict(payload=A + 8), -4), (dict(scales=A + 4), -4),
    (dict(p=_params(format=3)), -6), (dict(p=_params(format=-1)), -6),
    (dict(p=_params(mode=8)), -11), (dict(p=_params(mode=-1)), -11),
    (dict(p=_params(impl=7)), -8), (dict(p=_params(impl=-1)), -8),
    (dict(p=_params(layout=2)), -10), (dict(p=_params(layout=-1)), -10),
    (dict(p=_params(tau=0.0)), -9), (dict(p=_params(eps=-1.0)), -9), (dict(p=_params(tau=float("nan"))), -9),
])
def test_compress_rejects_bad_arguments(args, status):
    L = taco.lib()
    a = dict(x=A, rows=4, cols=512, p=_params(), payload=A, scales=A)
    a.update(args)
    pp = ctypes.byref(a["p"]) if a["p"] is not None else None
    assert L.taco_compress(a["x"], a["rows"], a["cols"], pp, a["payload"], a["scales"], None) == status


B0, B1, B2 = 0x100000, 0x200000, 0x300000      # fake pointers far enough apart for a [4, 512] tensor (4 KiB of bf16)


@pytest.mark.parametrize("x,payload,scales,layout", [
    (B0, B0, B1, 0),                    # output = input
    (B0, B0 + 4080, B1, 0),             # payload starts inside x (x is 4096 bytes)
    (B0 + 2032, B0, B1, 0),             # x starts inside the payload (2048 bytes)
    (B0, B1, B1 + 2032, 0),             # scales start inside the payload
    (B0, B1, B0 + 4080, 0),             # scales start inside x
    (B0, B0 + 4080, None, 1),           # interleaved records (2176 bytes) start inside x
    (B0 + 2160, B0, None, 1),           # x starts inside the records
])
def test_compress_rejects_overlapping_buffers(x, payload, scales, layout):
    L = taco.lib()
    p = _params(layout=layout)
    assert L.taco_compress(x, 4, 512, ctypes.byref(p), payload, scales, None) == -12


def test_decode_rejects_overlapping_buffers():
    L = taco.lib()
    p = _params()
    pl = (ctypes.c_void_p * 2)(B0, B1)
    sc = (ctypes.c_void_p * 2)(B2, B2 + 0x1000)
    # out (4096 bytes) over a payload (2048 bytes), over a scales region (128 bytes), just behind them: the last is fine,
    # so it is given a misaligned out to stop at the NEXT check instead of launching
    assert L.taco_decompress_sum(pl, sc, 2, 4, 512, ctypes.byref(p), B1 - 4080, None) == -12
    assert L.taco_decompress_sum(pl, sc, 2, 4, 512, ctypes.byref(p), B2 + 0x1000 + 112, None) == -12
    assert L.taco_decompress(B0, B2, 4, 512, ctypes.byref(p), B0 + 2032, None) == -12
    # the fused form: its outputs against the inputs and against each other
    assert L.taco_decompress_sum_compress(pl, sc, 2, 4, 512, ctypes.byref(p), B1 + 2032, B2 + 0x2000, None) == -12
    assert L.taco_decompress_sum_compress(pl, sc, 2, 4, 512, ctypes.byref(p), B2 + 0x2000, B2 + 0x2000 + 2032, None) == -12
    # inputs may repeat or overlap one another: the same payload twice passes the overlap test (and stops at k)
    same = (ctypes.c_void_p * 2)(B0, B0)
    assert L.taco_decompress_sum(same, sc, 17, 4, 512, ctypes.byref(p), B1, None) == -5


def _compress_items(entries):
    items = (taco.taco_compress_item * len(entries))()
    for i, (x, rows, cols, payload, scales) in enumerate(entries):
        items[i] = taco.taco_compress_item(x, rows, cols, payload, scales)
    return items


def test_compress_batch_rejects_bad_arguments():
    L = taco.lib()
    p = _params()
    ok = [(B0, 4, 512, B1, B2), (B0 + 0x10000, 4, 512, B1 + 0x10000, B2 + 0x10000)]
    assert L.taco_compress_batch(None, 1, ctypes.byref(p), None) == -1
    assert L.taco_compress_batch(_compress_items(ok), 0, ctypes.byref(p), None) == -13
    assert L.taco_compress_batch(_compress_items(ok * 17), 33, ctypes.byref(p), None) == -13
    assert L.taco_compress_batch(_compress_items(ok), 2, None, None) == -1
    assert L.taco_compress_batch(_compress_items(ok), 2, ctypes.byref(_params(block=100)), None) == -3
    assert L.taco_compress_batch(_compress_items(ok), 2, ctypes.byref(_params(tau=0.0)), None) == -9
    assert L.taco_compress_batch(_compress_items([ok[0], (0, 4, 512, B1, B2)]), 2, ctypes.byref(p), None) == -1
    assert L.taco_compress_batch(_compress_items([ok[0], (B0 + 0x10000, 0, 512, B1, B2)]), 2, ctypes.byref(p), None) == -2
    assert L.taco_compress_batch(_compress_items([ok[0], (B0 + 0x10000, 4, 512, B1 + 0x10008, B2 + 0x10000)]), 2, ctypes.byref(p), None) == -4
    # the second tensor's payload runs into the first tensor's; the second tensor's scales lie over the first one's input
    assert L.taco_compress_batch(_compress_items([ok[0], (B0 + 0x10000, 4, 512, B1 + 2032, B2 + 0x10000)]), 2, ctypes.byref(p), None) == -12
    assert L.taco_compress_batch(_compress_items([ok[0], (B0 + 0x10000, 4, 512, B1 + 0x10000, B0 + 16)]), 2, ctypes.byref(p), None) == -12


def test_decompress_sum_batch_rejects_bad_arguments():
    L = taco.lib()
    p = _params()
    pl = (ctypes.c_void_p * 2)(B0, B1)
    sc = (ctypes.c_void_p * 2)(B2, B2 + 0x1000)
    cast = lambda a: ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))

    def items(entries):
        arr = (taco.taco_decode_item * len(entries))()
        for i, e in enumerate(entries):
            arr[i] = taco.taco_decode_item(*e)
        return arr

    good = (cast(pl), cast(sc), 4, 512, B2 + 0x100000)
    assert L.taco_decompress_sum_batch(None, 1, 2, ctypes.byref(p), None) == -1
    assert L.taco_decompress_sum_batch(items([good]), 0, 2, ctypes.byref(p), None) == -13
    assert L.taco_decompress_sum_batch(items([good] * 33), 33, 2, ctypes.byref(p), None) == -13
    assert L.taco_decompress_sum_batch(items([good] * 9), 9, 16, ctypes.byref(p), None) == -13      # 144 payloads in all
    assert L.taco_decompress_sum_batch(items([good]), 1, 0, ctypes.byref(p), None) == -5
    assert L.taco_decompress_sum_batch(items([good]), 1, 17, ctypes.byref(p), None) == -5
    assert L.taco_decompress_sum_batch(items([good, (cast(pl), cast(sc), 4, 512, 0)]), 2, 2, ctypes.byref(p), None) == -1
    assert L.taco_decompress_sum_batch(items([good, (None, cast(sc), 4, 512, B2 + 0x200000)]), 2, 2, ctypes.byref(p), None) == -1
    assert L.taco_decompress_sum_batch(items([good, (cast(pl), cast(sc), -1, 512, B2 + 0x200000)]), 2, 2, ctypes.byref(p), None) == -2
    assert L.taco_decompress_sum_batch(items([good, (cast(pl), cast(sc), 4, 512, B2 + 0x200004)]), 2, 2, ctypes.byref(p), None) == -4
    # the second tensor's output over the first tensor's output, and over a payload
    assert L.taco_decompress_sum_batch(items([good, (cast(pl), cast(sc), 4, 512, B2 + 0x100000 + 4080)]), 2, 2, ctypes.byref(p), None) == -12
    assert L.taco_decompress_sum_batch(items([good, (cast(pl), cast(sc), 4, 512, B1 + 16)]), 2, 2, ctypes.byref(p), None) == -12


def test_fused_batch_rejects_bad_arguments():
    L = taco.lib()
    p = _params()
    pl = (ctypes.c_void_p * 2)(B0, B1)
    sc = (ctypes.c_void_p * 2)(B2, B2 + 0x1000)
    cast = lambda a: ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))

    def items(entries):
        arr = (taco.taco_recompress_item * len(entries))()
        for i, e in enumerate(entries):
            arr[i] = taco.taco_recompress_item(*e)
        return arr

    call = L.taco_decompress_sum_compress_batch
    good = (cast(pl), cast(sc), 4, 512, B2 + 0x100000, B2 + 0x180000)
    assert call(None, 1, 2, ctypes.byref(p), None) == -1
    assert call(items([good]), 0, 2, ctypes.byref(p), None) == -13
    assert call(items([good] * 33), 33, 2, ctypes.byref(p), None) == -13
    assert call(items([good]), 1, 17, ctypes.byref(p), None) == -5
    assert call(items([good]), 1, 2, ctypes.byref(_params(tau=0.0)), None) == -9            # the compress half needs tau > 0
    assert call(items([good, (cast(pl), cast(sc), 4, 512, 0, B2 + 0x190000)]), 2, 2, ctypes.byref(p), None) == -1
    assert call(items([good, (cast(pl), cast(sc), 4, 512, B2 + 0x110000, None)]), 2, 2, ctypes.byref(p), None) == -1
    assert call(items([good, (cast(pl), cast(sc), 4, 512, B2 + 0x110000, None)]), 2, 2, ctypes.byref(_params(layout=1)), None) != -1
    assert call(items([good, (cast(pl), cast(sc), 0, 512, B2 + 0x110000, B2 + 0x190000)]), 2, 2, ctypes.byref(p), None) == -2
    assert call(items([good, (cast(pl), cast(sc), 4, 512, B2 + 0x110008, B2 + 0x190000)]), 2, 2, ctypes.byref(p), None) == -4
    # the second tensor's payload over the first tensor's payload, and its scales over a source
    assert call(items([good, (cast(pl), cast(sc), 4, 512, B2 + 0x100000 + 2032, B2 + 0x190000)]), 2, 2, ctypes.byref(p), None) == -12
    assert call(items([good, (cast(pl), cast(sc), 4, 512, B2 + 0x110000, B0 + 16)]), 2, 2, ctypes.byref(p), None) == -12


@pytest.mark.parametrize("k,status", [(0, -5), (17, -5), (-1, -5)])
def test_decompress_sum_rejects_bad_k(k, status):
    L = taco.lib()
    arr = (ctypes.c_void_p * 17)(*([A] * 17))
    p = _params()
    assert L.taco_decompress_sum(arr, arr, k, 4, 512, ctypes.byref(p), A, None) == status


def test_interleaved_layout_needs_no_scales_pointer():
    """With records of codes + scalars the scales arguments are ignored; the calls below stop at the
    NEXT check (a misaligned payload), which shows the NULL scales pointers were accepted."""
    L = taco.lib()
    p = _params(layout=1)
    assert L.taco_compress(A, 4, 512, ctypes.byref(p), A + 8, None, None) == -4
    arr = (ctypes.c_void_p * 2)(A, A + 8)
    assert L.taco_decompress_sum(arr, None, 2, 4, 512, ctypes.byref(p), A, None) == -4
    assert L.taco_decompress_sum_compress(arr, None, 2, 4, 512, ctypes.byref(p), A, None, None) == -4
    split = _params(layout=0)
    assert L.taco_decompress_sum(arr, None, 2, 4, 512, ctypes.byref(split), A, None) == -1


def test_fused_rejects_bad_arguments():
    L = taco.lib()
    p = _params()
    arr = (ctypes.c_void_p * 2)(A, A)
    assert L.taco_decompress_sum_compress(arr, arr, 2, 4, 512, ctypes.byref(p), 0, A, None) == -1
    assert L.taco_decompress_sum_compress(arr, arr, 2, 4, 512, ctypes.byref(p), A, 0, None) == -1
    assert L.taco_decompress_sum_compress(arr, arr, 0, 4, 512, ctypes.byref(p), A, A, None) == -5
    assert L.taco_decompress_sum_compress(arr, arr, 2, 0, 512, ctypes.byref(p), A, A, None) == -2
    assert L.taco_decompress_sum_compress(arr, arr, 2, 4, 512, ctypes.byref(p), A + 4, A, None) == -4
    bad = _params(tau=-1.0)
    assert L.taco_decompress_sum_compress(arr, arr, 2, 4, 512, ctypes.byref(bad), A, A, None) == -9


def test_debug_traffic_rejects_bad_arguments():
    L = taco.lib()
    arr = (ctypes.c_void_p * 2)(A, A)
    assert L.taco_debug_traffic(None, 1, 256, A, 136, 4, None) == -1
    assert L.taco_debug_traffic(arr, 1, 256, 0, 136, 4, None) == -1
    assert L.taco_debug_traffic(arr, 0, 256, A, 136, 4, None) == -5
    assert L.taco_debug_traffic(arr, 17, 256, A, 136, 4, None) == -5
    assert L.taco_debug_traffic(arr, 1, 0, A, 136, 4, None) == -2
    assert L.taco_debug_traffic(arr, 1, 257, A, 136, 4, None) == -2
    assert L.taco_debug_traffic(arr, 1, 256, A, 300, 4, None) == -2
    assert L.taco_debug_traffic(arr, 1, 256, A, 136, 0, None) == -2
    assert L.taco_debug_traffic(arr, 2, 256, A + 8, 136, 4, None) == -4
    bad = (ctypes.c_void_p * 2)(A, A + 4)
    assert L.taco_debug_traffic(bad, 2, 256, A, 136, 4, None) == -4
    null = (ctypes.c_void_p * 2)(A, 0)
    assert L.taco_debug_traffic(null, 2, 256, A, 136, 4, None) == -1


def test_decompress_rejects_bad_arguments():
    L = taco.lib()
    p = _params()
    arr = (ctypes.c_void_p * 2)(A, 0)
    assert L.taco_decompress(0, A, 4, 512, ctypes.byref(p), A, None) == -1
    assert L.taco_decompress(A, A, 4, 512, ctypes.byref(p), 0, None) == -1
    assert L.taco_decompress(A, A, 4, 512, ctypes.byref(p), A + 2, None) == -4
    assert L.taco_decompress_sum(arr, arr, 2, 4, 512, ctypes.byref(p), A, None) == -1     # null entry
    assert L.taco_decompress_sum(None, arr, 1, 4, 512, ctypes.byref(p), A, None) == -1
    assert L.taco_debug_cvt_e4m3(0, 4, A, None) == -1
    assert L.taco_debug_cvt_e4m3(A, 0, A, None) == -2
    assert L.taco_debug_cvt_e4m3(A, (1 << 31) + 1, A, None) == -2
    with pytest.raises(taco.TacoError):
        taco._check(-3, "x")


def test_binding_rejects_tensors_that_are_not_gpu_buffers():
    """The Python binding checks device, dtype, contiguity and size before it hands a pointer to the library."""
    import torch
    x = torch.zeros(4, 512, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="CUDA"):
        taco.taco_compress(x)
    with pytest.raises(ValueError, match="CUDA"):
        taco.taco_decompress(torch.zeros(2048, dtype=torch.uint8), torch.zeros(16, 2), (4, 512))
    with pytest.raises(ValueError, match="between 1 and 16"):
        taco.taco_decompress_sum([], [], (4, 512))
    with pytest.raises(ValueError, match="CUDA"):
        taco.taco_debug_copy(x, x.clone())


def test_binding_size_formula_matches_the_library():
    for n in (0, -3, 1, 31, 32, 33, 127, 128, 129, 2048, 2049, 10 ** 9 + 7, 2 ** 36, 2 ** 36 + 1):
        for b in (16, 32, 64, 100, 128, 256, 512, 1024):
            assert taco._sizes(n, b) == (taco.taco_payload_bytes(n, b), taco.taco_scales_bytes(n, b)), (n, b)
