"""CPU-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before queuing anything (no
compute call is made here; pointers are fake and never dereferenced)."""
import ctypes as C
import os
import re

import pytest

from paper_2410_00531_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000          # a non-null, 16-byte aligned address that is never touched


def _header_functions():
    txt = open(os.path.join(ROOT, "include", "tpi.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(tpi_[a-z_0-9]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    names = _header_functions()
    assert set(names) == set(B.EXPORTED), (names, B.EXPORTED)
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None
    assert B.tpi_abi_version() == 1


def test_struct_layouts_match_the_header():
    assert C.sizeof(B.tpi_shard_cfg) == 36
    assert C.sizeof(B.tpi_layer_weights) == 56
    assert C.sizeof(B.tpi_kv_layer) == 16
    assert C.sizeof(B.tpi_window_block) == 32
    assert C.sizeof(B.tpi_window_slots) == 24
    assert C.sizeof(B.tpi_window_file_block) == 40


def _w():
    return B.tpi_layer_weights(*([FAKE] * 7))


def _code(fn, *a, **k):
    with pytest.raises(B.TpiError) as ei:
        fn(*a, **k)
    return ei.value.code


def test_workspace_bytes():
    cfg = B.make_cfg(8192, 8, 1, 128, 3584, 1100)
    n = B.tpi_workspace_bytes(cfg, 1)
    # q + split maxima and sums + split outputs + merged output + activation + tickets, in floats
    assert n == 4 * (1024 + 2 * 8 * 32 + 8 * 32 * 128 + 1024 + 3584 + 4)
    assert B.tpi_workspace_bytes(B.make_cfg(8192, 8, 3, 128, 3584, 1100), 1) == 0
    assert B.tpi_workspace_bytes(cfg, 0) == 0


def test_rows_longer_than_the_stages_are_built_for_are_refused():
    kv = B.tpi_kv_layer(FAKE, FAKE)
    for cfg in (B.make_cfg(16388, 2, 1, 64, 128, 8), B.make_cfg(256, 2, 1, 64, 16388, 8), B.make_cfg(256, 129, 1, 128, 64, 8)):
        assert _code(B.tpi_shard_layer_decode, cfg, _w(), kv, 3, B.TPI_PHASE_ATTN, FAKE, FAKE, FAKE, stream=0) == B.TPI_EUNSUPPORTED


def test_decode_argument_errors():
    good = B.make_cfg(256, 2, 2, 64, 344, 24)
    kv = B.tpi_kv_layer(FAKE, FAKE)
    call = lambda cfg, pos=3, phase=B.TPI_PHASE_ATTN, w=None, kvv=kv, h=FAKE, out=FAKE, ws=FAKE: \
        B.tpi_shard_layer_decode(cfg, w or _w(), kvv, pos, phase, h, out, ws, stream=0)
    assert _code(call, good, pos=-1) == B.TPI_EINVAL
    assert _code(call, good, pos=24) == B.TPI_EINVAL
    assert _code(call, good, phase=7) == B.TPI_EINVAL
    assert _code(call, good, h=None) == B.TPI_EINVAL
    assert _code(call, good, out=None) == B.TPI_EINVAL
    assert _code(call, good, ws=None) == B.TPI_EINVAL
    assert _code(call, good, kvv=None) == B.TPI_EINVAL
    assert _code(call, good, kvv=B.tpi_kv_layer(FAKE, None)) == B.TPI_EINVAL
    wbad = _w(); wbad.w_o = None
    assert _code(call, good, w=wbad) == B.TPI_EINVAL
    assert _code(call, B.make_cfg(256, 3, 2, 64, 344, 24)) == B.TPI_EINVAL       # heads not a multiple
    assert _code(call, B.make_cfg(256, 2, 2, 63, 344, 24)) == B.TPI_EINVAL       # odd head size
    assert _code(call, B.make_cfg(0, 2, 2, 64, 344, 24)) == B.TPI_EINVAL
    assert _code(call, B.make_cfg(256, 2, 2, 64, 344, 0)) == B.TPI_EINVAL
    assert _code(call, B.make_cfg(256, 2, 2, 64, 344, 24, dtype=5)) == B.TPI_EINVAL
    assert _code(call, B.make_cfg(256, 2, 2, 66, 344, 24)) == B.TPI_EUNSUPPORTED  # not a multiple of 4
    assert _code(call, B.make_cfg(256, 2, 2, 512, 344, 24)) == B.TPI_EUNSUPPORTED
    assert _code(call, B.make_cfg(256, 2, 2, 64, 344, 24, dtype=B.TPI_BF16)) == B.TPI_EUNSUPPORTED
    assert _code(call, good, h=FAKE + 4) == B.TPI_EUNSUPPORTED                   # misaligned
    assert "aligned" in B.tpi_last_error()
    # batched variant: shard count limits
    n = B.TPI_MAX_BATCH_SHARDS + 1
    assert _code(B.tpi_shards_layer_decode, good, [_w()] * n, [kv] * n, 3, B.TPI_PHASE_ATTN, FAKE,
                 [FAKE] * n, [FAKE] * n, stream=0) == B.TPI_EINVAL
    # batched variant with the reduce folded in
    fused = lambda k=2, out=FAKE, h=FAKE, ws=FAKE, pos=3: B.tpi_shards_layer_decode_reduce(
        good, [_w()] * k, [kv] * k, pos, B.TPI_PHASE_ATTN, h, out, [ws] * k, stream=0)
    assert _code(fused, k=n) == B.TPI_EINVAL
    assert _code(fused, out=None) == B.TPI_EINVAL
    assert _code(fused, h=None) == B.TPI_EINVAL
    assert _code(fused, ws=None) == B.TPI_EINVAL
    assert _code(fused, pos=24) == B.TPI_EINVAL
    assert _code(fused, out=FAKE + 4) == B.TPI_EUNSUPPORTED
    # out must not overlap h_in: other workgroups still read h_in while a workgroup writes its rows of out
    assert _code(fused, out=FAKE, h=FAKE) == B.TPI_EINVAL and "overlaps" in B.tpi_last_error()
    assert _code(fused, out=FAKE + 256 * 4 - 16, h=FAKE) == B.TPI_EINVAL and "overlaps" in B.tpi_last_error()


def test_star_reduce_and_prefill_argument_errors():
    assert _code(B.tpi_star_reduce, [], None, FAKE, length=4, stream=0) == B.TPI_EINVAL
    assert _code(B.tpi_star_reduce, [FAKE], None, FAKE, length=-1, stream=0) == B.TPI_EINVAL
    assert _code(B.tpi_star_reduce, [FAKE, None], None, FAKE, length=4, stream=0) == B.TPI_EINVAL
    assert _code(B.tpi_star_reduce, [FAKE], None, None, length=4, stream=0) == B.TPI_EINVAL
    assert _code(B.tpi_star_reduce, [FAKE] * 65, None, FAKE, length=4, stream=0) == B.TPI_EUNSUPPORTED
    cfg = B.make_cfg(256, 2, 2, 64, 344, 24, dtype=B.TPI_BF16)
    kv = B.tpi_kv_layer(FAKE, FAKE)
    pre = lambda c, pos0, n: B.tpi_shard_layer_prefill(c, _w(), kv, pos0, n, B.TPI_PHASE_ATTN, FAKE, FAKE,
                                                       FAKE, stream=0)
    assert _code(pre, cfg, 20, 5) == B.TPI_EINVAL
    assert _code(pre, cfg, -1, 5) == B.TPI_EINVAL
    assert _code(pre, cfg, 0, 0) == B.TPI_EINVAL
    assert _code(pre, B.make_cfg(256, 2, 2, 64, 344, 24), 0, 4) == B.TPI_EUNSUPPORTED   # fp32 prefill
    # per-shard pointers are checked before anything is queued
    assert _code(B.tpi_shard_layer_prefill, cfg, _w(), B.tpi_kv_layer(FAKE, None), 0, 4, B.TPI_PHASE_ATTN, FAKE, FAKE,
                 FAKE, stream=0) == B.TPI_EINVAL
    assert _code(B.tpi_shard_layer_prefill, cfg, _w(), kv, 0, 4, B.TPI_PHASE_ATTN, FAKE, None, FAKE, stream=0) == B.TPI_EINVAL
    assert _code(B.tpi_shard_layer_prefill, cfg, _w(), kv, 0, 4, B.TPI_PHASE_ATTN, FAKE, FAKE + 4, FAKE,
                 stream=0) == B.TPI_EUNSUPPORTED
    # all shards of a phase per call: shard count limits, a null entry in the arrays
    for n in (0, B.TPI_MAX_BATCH_SHARDS + 1):
        assert _code(B.tpi_shards_layer_prefill, cfg, [_w()] * n, [kv] * n, 0, 4, B.TPI_PHASE_ATTN, FAKE, [FAKE] * n,
                     [FAKE] * n, stream=0) == B.TPI_EINVAL
    assert _code(B.tpi_shards_layer_prefill, cfg, [_w()] * 2, [kv] * 2, 0, 4, B.TPI_PHASE_ATTN, FAKE, [FAKE, None],
                 [FAKE] * 2, stream=0) == B.TPI_EINVAL
    assert "shard 1" in B.tpi_last_error()
    assert _code(B.tpi_shards_layer_prefill, cfg, [_w()] * 2, None, 0, 4, B.TPI_PHASE_ATTN, FAKE, [FAKE] * 2,
                 [FAKE] * 2, stream=0) == B.TPI_EINVAL


def test_window_argument_errors_without_a_device():
    h = C.c_void_p()
    lib = B.lib()
    arr = (C.c_void_p * 2)(FAKE, FAKE)
    assert lib.tpi_window_create(C.byref(h), 0, 1, 16, arr, FAKE) == B.TPI_EINVAL
    assert lib.tpi_window_create(C.byref(h), 2, 0, 16, arr, FAKE) == B.TPI_EINVAL
    assert lib.tpi_window_create(C.byref(h), 2, 1, 0, arr, FAKE) == B.TPI_EINVAL
    assert lib.tpi_window_create(C.byref(h), 2, 1, 16, None, FAKE) == B.TPI_EINVAL
    arr2 = (C.c_void_p * 2)(FAKE, None)
    assert lib.tpi_window_create(C.byref(h), 2, 1, 16, arr2, FAKE) == B.TPI_EINVAL
    # block-granular creation: every malformed description is refused before any HIP call
    blk = lambda host=FAKE, nbytes=16, cls=0, retained=0, resident=None: B.tpi_window_block(host, nbytes, cls, retained, resident)
    one_class = (B.tpi_window_slots * 1)(B.tpi_window_slots(FAKE, 16, 2))
    mk = lambda *bs: (B.tpi_window_block * len(bs))(*bs)
    cb = lib.tpi_window_create_blocks
    assert cb(C.byref(h), 0, mk(blk()), 1, one_class) == B.TPI_EINVAL
    assert cb(C.byref(h), 1, mk(blk()), 0, one_class) == B.TPI_EINVAL
    assert cb(C.byref(h), 1, None, 1, one_class) == B.TPI_EINVAL
    assert cb(C.byref(h), 1, mk(blk()), 1, None) == B.TPI_EINVAL
    assert cb(C.byref(h), 1, mk(blk(host=None)), 1, one_class) == B.TPI_EINVAL
    assert cb(C.byref(h), 1, mk(blk(nbytes=0)), 1, one_class) == B.TPI_EINVAL
    assert cb(C.byref(h), 1, mk(blk(nbytes=17)), 1, one_class) == B.TPI_EINVAL          # larger than its slot
    assert b"do not fit" in lib.tpi_last_error()
    assert cb(C.byref(h), 1, mk(blk(cls=1)), 1, one_class) == B.TPI_EINVAL              # class out of range
    assert cb(C.byref(h), 1, mk(blk(retained=1)), 1, one_class) == B.TPI_EINVAL         # retained, no home
    assert cb(C.byref(h), 1, mk(blk()), 1, (B.tpi_window_slots * 1)(B.tpi_window_slots(FAKE, 16, 0))) == B.TPI_EINVAL
    assert cb(C.byref(h), 1, mk(blk()), 1, (B.tpi_window_slots * 1)(B.tpi_window_slots(None, 16, 1))) == B.TPI_EINVAL
    # file tier: the description and the files are checked before anything is created on a device
    fblk = lambda path=b"/nonexistent/tpi_block", nbytes=16: B.tpi_window_file_block(path, 0, nbytes, 0, 0, None)
    fmk = lambda *bs: (B.tpi_window_file_block * len(bs))(*bs)
    cf = lib.tpi_window_create_files
    assert cf(C.byref(h), 1, fmk(fblk()), 1, one_class, 0, 1) == B.TPI_EINVAL            # no staging buffer
    assert cf(C.byref(h), 1, fmk(fblk()), 1, one_class, 2, 0) == B.TPI_EINVAL            # no reader
    assert cf(C.byref(h), 1, fmk(fblk(path=None)), 1, one_class, 2, 1) == B.TPI_EINVAL
    assert cf(C.byref(h), 1, fmk(fblk()), 1, one_class, 2, 1) == B.TPI_EINVAL
    assert b"cannot open" in lib.tpi_last_error()
    assert cf(C.byref(h), 0, fmk(fblk()), 1, one_class, 2, 1) == B.TPI_EINVAL
    assert cf(C.byref(h), 1, None, 1, one_class, 2, 1) == B.TPI_EINVAL
    assert lib.tpi_window_read_stats(None, None) == B.TPI_EINVAL
    assert lib.tpi_window_prefetch(None, 0) == B.TPI_EINVAL
    assert lib.tpi_window_destroy(None) == B.TPI_EINVAL


def test_whole_token_kernel_is_reported_unavailable():
    cfg = B.make_cfg(256, 2, 2, 64, 344, 24)
    h = C.c_void_p()
    w = (B.tpi_layer_weights * 1)(_w())
    kv = (B.tpi_kv_layer * 1)(B.tpi_kv_layer(FAKE, FAKE))
    rc = B.lib().tpi_decoder_create(C.byref(h), C.byref(cfg), 1, w, kv, 1, 0, None, None, 0x10000, 0)
    assert rc == B.TPI_EUNSUPPORTED and "switched off" in B.tpi_last_error()
    assert B.lib().tpi_decoder_create(C.byref(h), C.byref(cfg), 0, w, kv, 1, 0, None, None, 0x10000, 0) == B.TPI_EINVAL


def test_token_ends_argument_errors_without_a_device():
    lib = B.lib()
    assert lib.tpi_embed_token(None, 10, 8, 0, FAKE, None) == B.TPI_EINVAL
    assert lib.tpi_embed_token(FAKE, 10, 8, 10, FAKE, None) == B.TPI_EINVAL       # token outside the vocabulary
    assert lib.tpi_embed_token(FAKE, 10, 8, -1, FAKE, None) == B.TPI_EINVAL
    assert lib.tpi_embed_token(FAKE, 0, 8, 0, FAKE, None) == B.TPI_EINVAL
    head = lambda norm=FAKE, w=FAKE, v=10, h=8, eps=1e-5, x=FAKE, out=FAKE: lib.tpi_lm_head(norm, w, v, h, eps, x, out, None)
    assert head(norm=None) == B.TPI_EINVAL and head(out=None) == B.TPI_EINVAL
    assert head(v=0) == B.TPI_EINVAL
    assert head(h=6) == B.TPI_EINVAL and head(h=0) == B.TPI_EINVAL
    assert head(eps=0.0) == B.TPI_EINVAL
    assert head(h=16388) == B.TPI_EUNSUPPORTED
    assert head(w=FAKE + 4) == B.TPI_EUNSUPPORTED
    assert lib.tpi_next_token(None, 10, 0.5, None, FAKE, None) == B.TPI_EINVAL
    assert lib.tpi_next_token(FAKE, 10, 0.5, None, None, None) == B.TPI_EINVAL
    assert lib.tpi_next_token(FAKE, 0, 0.5, None, FAKE, None) == B.TPI_EINVAL
    assert lib.tpi_next_token(FAKE, 10, 1.0, None, FAKE, None) == B.TPI_EINVAL
    assert lib.tpi_next_token(FAKE, 10, float("nan"), None, FAKE, None) == B.TPI_EINVAL



def test_prefill_concurrency_hint_arguments():
    lib = B.lib()
    assert lib.tpi_set_prefill_concurrency(0) == B.TPI_EINVAL
    assert lib.tpi_set_prefill_concurrency(B.TPI_MAX_BATCH_SHARDS + 1) == B.TPI_EINVAL
    assert b"n_calls" in lib.tpi_last_error()
    assert lib.tpi_set_prefill_concurrency(2) == B.TPI_OK
    assert lib.tpi_set_prefill_concurrency(1) == B.TPI_OK
