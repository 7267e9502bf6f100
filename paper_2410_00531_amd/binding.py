"""ctypes binding of libtpi.so: the same names as include/tpi.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels;
there is no fallback: a missing library raises.

Tensors are torch CUDA tensors (PyTorch-ROCm is used for device memory and
streams); the functions take their data pointers and the current stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtpi.so")

TPI_OK, TPI_EINVAL, TPI_EUNSUPPORTED, TPI_ERUNTIME, TPI_ESTATE = 0, -1, -2, -3, -4
TPI_F32, TPI_BF16 = 0, 1
TPI_PHASE_ATTN, TPI_PHASE_FFN = 1, 2
TPI_MAX_REDUCE_RANKS = 64
TPI_MAX_BATCH_SHARDS = 16

EXPORTED = (
    "tpi_workspace_bytes", "tpi_shard_layer_decode", "tpi_shards_layer_decode", "tpi_set_prefill_concurrency", "tpi_shards_layer_prefill",
    "tpi_shard_layer_decode_reduce", "tpi_shards_layer_decode_reduce", "tpi_shard_layer_decode_static",
    "tpi_shard_layer_prefill", "tpi_star_reduce", "tpi_star_reduce_bf16", "tpi_window_create",
    "tpi_window_create_blocks", "tpi_window_create_files", "tpi_window_read_stats", "tpi_window_prefetch",
    "tpi_embed_token", "tpi_lm_head", "tpi_next_token",
    "tpi_window_acquire", "tpi_window_release", "tpi_window_destroy", "tpi_window_copy_stats",
    "tpi_last_error", "tpi_abi_version", "tpi_prof_enable", "tpi_prof_read",
    "tpi_decoder_workspace_bytes", "tpi_decoder_create", "tpi_decoder_token", "tpi_decoder_status",
    "tpi_decoder_grid", "tpi_decoder_destroy",
    "tpi_sim_create", "tpi_sim_stream", "tpi_sim_read", "tpi_sim_run", "tpi_sim_hash", "tpi_sim_destroy",
    "tpi_sim_set_copy_rate", "tpi_sim_stream_time", "tpi_probe_handover", "tpi_probe_gemm_loop", "tpi_kv_widen", "tpi_window_calibrate",
    "tpi_window_create_blocks_sim", "tpi_window_create_files_sim",
)
TPI_STAGE_NONE, TPI_STAGE_QKV, TPI_STAGE_ATTN, TPI_STAGE_OPROJ = 0, 1, 2, 3
TPI_STAGE_GATE_UP, TPI_STAGE_DOWN, TPI_STAGE_REDUCE, TPI_STAGE_PREFILL_GEMM = 4, 5, 6, 7
TPI_STAGE_TOKEN = 8


class TpiError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libtpi error {code}: {msg}")
        self.code = code


class tpi_shard_cfg(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_local", C.c_int32), ("n_kv_local", C.c_int32),
                ("head_dim", C.c_int32), ("ffn_local", C.c_int32), ("max_seq", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32)]


class tpi_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate", "w_up", "w_down")]


class tpi_kv_layer(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p)]


class tpi_window_block(C.Structure):
    _fields_ = [("host", C.c_void_p), ("bytes", C.c_size_t), ("slot_class", C.c_int32),
                ("retained", C.c_int32), ("resident", C.c_void_p)]


class tpi_window_file_block(C.Structure):
    _fields_ = [("path", C.c_char_p), ("offset", C.c_uint64), ("bytes", C.c_size_t), ("slot_class", C.c_int32),
                ("retained", C.c_int32), ("resident", C.c_void_p)]


class tpi_window_slots(C.Structure):
    _fields_ = [("base", C.c_void_p), ("slot_bytes", C.c_size_t), ("n_slots", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Loads libtpi.so (built in-tree by ``build.build_lib``); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first "
                               "(python -m paper_2410_00531_amd.build); there is no fallback path")
        l = C.CDLL(LIB_PATH)
        l.tpi_workspace_bytes.restype = C.c_size_t
        l.tpi_workspace_bytes.argtypes = [C.POINTER(tpi_shard_cfg), C.c_int32]
        l.tpi_last_error.restype = C.c_char_p
        l.tpi_abi_version.restype = C.c_int
        l.tpi_shard_layer_decode.restype = C.c_int
        l.tpi_shard_layer_decode.argtypes = [C.POINTER(tpi_shard_cfg), C.POINTER(tpi_layer_weights),
                                             C.POINTER(tpi_kv_layer), C.c_int32, C.c_int, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
        l.tpi_shard_layer_decode_static.restype = C.c_int
        l.tpi_shard_layer_decode_static.argtypes = [C.POINTER(tpi_shard_cfg), C.POINTER(tpi_layer_weights),
                                                    C.POINTER(tpi_kv_layer), C.c_int32, C.c_int, C.c_void_p,
                                                    C.c_void_p, C.c_void_p]
        l.tpi_shard_layer_decode_reduce.restype = C.c_int
        l.tpi_shard_layer_decode_reduce.argtypes = [C.POINTER(tpi_shard_cfg), C.POINTER(tpi_layer_weights),
                                                    C.POINTER(tpi_kv_layer), C.c_int32, C.c_int, C.c_void_p,
                                                    C.c_int32, C.c_int32, C.POINTER(C.c_void_p), C.c_void_p,
                                                    C.c_void_p, C.c_void_p]
        l.tpi_shards_layer_decode.restype = C.c_int
        l.tpi_shards_layer_decode.argtypes = [C.POINTER(tpi_shard_cfg), C.c_int32,
                                              C.POINTER(tpi_layer_weights), C.POINTER(tpi_kv_layer),
                                              C.c_int32, C.c_int, C.c_void_p, C.POINTER(C.c_void_p),
                                              C.POINTER(C.c_void_p), C.c_void_p]
        l.tpi_shards_layer_decode_reduce.restype = C.c_int
        l.tpi_shards_layer_decode_reduce.argtypes = [C.POINTER(tpi_shard_cfg), C.c_int32,
                                                     C.POINTER(tpi_layer_weights), C.POINTER(tpi_kv_layer),
                                                     C.c_int32, C.c_int, C.c_void_p, C.c_void_p,
                                                     C.POINTER(C.c_void_p), C.c_void_p]
        l.tpi_shard_layer_prefill.restype = C.c_int
        l.tpi_shard_layer_prefill.argtypes = [C.POINTER(tpi_shard_cfg), C.POINTER(tpi_layer_weights),
                                              C.POINTER(tpi_kv_layer), C.c_int32, C.c_int32, C.c_int,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.tpi_shards_layer_prefill.restype = C.c_int
        l.tpi_shards_layer_prefill.argtypes = [C.POINTER(tpi_shard_cfg), C.c_int32, C.POINTER(tpi_layer_weights),
                                               C.POINTER(tpi_kv_layer), C.c_int32, C.c_int32, C.c_int, C.c_void_p,
                                               C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p]
        l.tpi_set_prefill_concurrency.restype = C.c_int
        l.tpi_set_prefill_concurrency.argtypes = [C.c_int32]
        l.tpi_star_reduce.restype = C.c_int
        l.tpi_star_reduce.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_int64, C.c_void_p,
                                      C.c_void_p, C.c_void_p]
        l.tpi_star_reduce_bf16.restype = C.c_int
        l.tpi_star_reduce_bf16.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_int64, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p]
        l.tpi_window_create.restype = C.c_int
        l.tpi_window_create.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.c_size_t,
                                        C.POINTER(C.c_void_p), C.c_void_p]
        l.tpi_window_create_blocks.restype = C.c_int
        l.tpi_window_create_blocks.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.POINTER(tpi_window_block),
                                               C.c_int32, C.POINTER(tpi_window_slots)]
        l.tpi_window_create_blocks_sim.restype = C.c_int
        l.tpi_window_create_blocks_sim.argtypes = [C.POINTER(C.c_void_p), C.c_void_p, C.c_int32, C.POINTER(tpi_window_block),
                                                   C.c_int32, C.POINTER(tpi_window_slots)]
        l.tpi_window_create_files_sim.restype = C.c_int
        l.tpi_window_create_files_sim.argtypes = [C.POINTER(C.c_void_p), C.c_void_p, C.c_int32,
                                                  C.POINTER(tpi_window_file_block), C.c_int32,
                                                  C.POINTER(tpi_window_slots), C.c_int32, C.c_int32]
        l.tpi_window_create_files.restype = C.c_int
        l.tpi_window_create_files.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.POINTER(tpi_window_file_block),
                                              C.c_int32, C.POINTER(tpi_window_slots), C.c_int32, C.c_int32]
        l.tpi_window_read_stats.restype = C.c_int
        l.tpi_window_read_stats.argtypes = [C.c_void_p, C.POINTER(C.c_double)]
        for name in ("tpi_window_prefetch",):
            getattr(l, name).restype = C.c_int
            getattr(l, name).argtypes = [C.c_void_p, C.c_int32]
        l.tpi_window_acquire.restype = C.c_int
        l.tpi_window_acquire.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_void_p)]
        l.tpi_window_release.restype = C.c_int
        l.tpi_window_release.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        l.tpi_window_destroy.restype = C.c_int
        l.tpi_window_destroy.argtypes = [C.c_void_p]
        l.tpi_window_copy_stats.restype = C.c_int
        l.tpi_window_copy_stats.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
        l.tpi_embed_token.restype = C.c_int
        l.tpi_embed_token.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        l.tpi_lm_head.restype = C.c_int
        l.tpi_lm_head.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p,
                                  C.c_void_p]
        l.tpi_next_token.restype = C.c_int
        l.tpi_next_token.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
        l.tpi_prof_enable.restype = C.c_int
        l.tpi_prof_enable.argtypes = [C.c_int, C.c_int32]
        l.tpi_prof_read.restype = C.c_int
        l.tpi_prof_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        l.tpi_decoder_workspace_bytes.restype = C.c_size_t
        l.tpi_decoder_workspace_bytes.argtypes = [C.POINTER(tpi_shard_cfg), C.c_int32]
        l.tpi_decoder_create.restype = C.c_int
        l.tpi_decoder_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(tpi_shard_cfg), C.c_int32,
                                         C.POINTER(tpi_layer_weights), C.POINTER(tpi_kv_layer), C.c_int32,
                                         C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p,
                                         C.c_void_p]
        l.tpi_decoder_token.restype = C.c_int
        l.tpi_decoder_token.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        l.tpi_decoder_status.restype = C.c_int
        l.tpi_decoder_status.argtypes = [C.c_void_p, C.c_void_p]
        l.tpi_decoder_grid.restype = C.c_int
        l.tpi_decoder_grid.argtypes = [C.c_void_p]
        l.tpi_decoder_destroy.restype = C.c_int
        l.tpi_decoder_destroy.argtypes = [C.c_void_p]
        _lib = l
    return _lib


def _check(rc: int) -> None:
    if rc != TPI_OK:
        raise TpiError(rc, lib().tpi_last_error().decode())


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_cfg(hidden, n_q_local, n_kv_local, head_dim, ffn_local, max_seq, rms_eps=1e-5,
             rope_base=10000.0, dtype=TPI_F32) -> tpi_shard_cfg:
    return tpi_shard_cfg(hidden, n_q_local, n_kv_local, head_dim, ffn_local, max_seq, rms_eps,
                         rope_base, dtype)


def make_weights(w) -> tpi_layer_weights:
    """w: mapping with the seven tensors (torch tensors or raw device addresses)."""
    return tpi_layer_weights(*[_ptr(w.get(n)) for n, _ in tpi_layer_weights._fields_])


def make_kv(k, v) -> tpi_kv_layer:
    return tpi_kv_layer(_ptr(k), _ptr(v))


def tpi_abi_version() -> int:
    return int(lib().tpi_abi_version())


def tpi_last_error() -> str:
    return lib().tpi_last_error().decode()


def tpi_set_prefill_concurrency(n_calls: int) -> None:
    _check(lib().tpi_set_prefill_concurrency(int(n_calls)))


def tpi_workspace_bytes(cfg: tpi_shard_cfg, n_tokens: int = 1) -> int:
    return int(lib().tpi_workspace_bytes(C.byref(cfg), n_tokens))


def tpi_shard_layer_decode(cfg, weights: tpi_layer_weights, kv: Optional[tpi_kv_layer], pos: int,
                           phase: int, h_in, partial_out, workspace, stream=None) -> None:
    _check(lib().tpi_shard_layer_decode(C.byref(cfg), C.byref(weights),
                                        C.byref(kv) if kv is not None else None, pos, phase,
                                        _ptr(h_in), _ptr(partial_out), _ptr(workspace), _stream(stream)))


def tpi_kv_widen(src_k, src_v, dst_k, dst_v, n_slots: int, stream=None) -> None:
    """src_*: bf16 caches [n_kv][src_max_seq][d]; dst_*: fp32 caches [n_kv][dst_max_seq][d] (torch tensors)."""
    l = lib()
    l.tpi_kv_widen.restype = C.c_int
    l.tpi_kv_widen.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(tpi_kv_layer), C.c_int32,
                               C.POINTER(tpi_kv_layer), C.c_int32, C.c_void_p]
    n_kv, src_seq, d = src_k.shape
    src, dst = make_kv(src_k, src_v), make_kv(dst_k, dst_v)
    _check(l.tpi_kv_widen(n_kv, d, n_slots, C.byref(src), src_seq, C.byref(dst), dst_k.shape[1], _stream(stream)))


def tpi_shard_layer_decode_static(cfg, weights: tpi_layer_weights, kv: Optional[tpi_kv_layer], pos: int,
                                  phase: int, h_in, partial_out, stream=None) -> None:
    _check(lib().tpi_shard_layer_decode_static(C.byref(cfg), C.byref(weights),
                                               C.byref(kv) if kv is not None else None, pos, phase,
                                               _ptr(h_in), _ptr(partial_out), _stream(stream)))


def tpi_shard_layer_decode_reduce(cfg, weights: tpi_layer_weights, kv: Optional[tpi_kv_layer], pos: int, phase: int,
                                  h_in, rank: int, partials, out, workspace, stream=None) -> None:
    """partials: sequence of n_ranks tensors / addresses (entry `rank` is ignored) or a prepared C array."""
    if isinstance(partials, C.Array):
        arr, n = partials, len(partials)
    else:
        n = len(partials)
        arr = (C.c_void_p * n)(*[(_ptr(p) if i != rank else None) for i, p in enumerate(partials)])
    _check(lib().tpi_shard_layer_decode_reduce(C.byref(cfg), C.byref(weights),
                                               C.byref(kv) if kv is not None else None, pos, phase, _ptr(h_in),
                                               n, rank, arr, _ptr(out), _ptr(workspace), _stream(stream)))


def tpi_shards_layer_decode(cfg, weights: Sequence[tpi_layer_weights],
                            kvs: Optional[Sequence[tpi_kv_layer]], pos: int, phase: int, h_in,
                            partial_outs, workspaces, stream=None) -> None:
    n = len(weights)
    warr = weights if isinstance(weights, C.Array) else (tpi_layer_weights * n)(*weights)
    if kvs is None:
        karr = None
    else:
        karr = kvs if isinstance(kvs, C.Array) else (tpi_kv_layer * n)(*kvs)
    parr = partial_outs if isinstance(partial_outs, C.Array) else (C.c_void_p * n)(*[_ptr(p) for p in partial_outs])
    wsarr = workspaces if isinstance(workspaces, C.Array) else (C.c_void_p * n)(*[_ptr(p) for p in workspaces])
    _check(lib().tpi_shards_layer_decode(C.byref(cfg), n, warr, karr, pos, phase, _ptr(h_in), parr,
                                         wsarr, _stream(stream)))


def tpi_shards_layer_decode_reduce(cfg, weights: Sequence[tpi_layer_weights],
                                   kvs: Optional[Sequence[tpi_kv_layer]], pos: int, phase: int, h_in, out,
                                   workspaces, stream=None) -> None:
    n = len(weights)
    warr = weights if isinstance(weights, C.Array) else (tpi_layer_weights * n)(*weights)
    if kvs is None:
        karr = None
    else:
        karr = kvs if isinstance(kvs, C.Array) else (tpi_kv_layer * n)(*kvs)
    wsarr = workspaces if isinstance(workspaces, C.Array) else (C.c_void_p * n)(*[_ptr(p) for p in workspaces])
    _check(lib().tpi_shards_layer_decode_reduce(C.byref(cfg), n, warr, karr, pos, phase, _ptr(h_in), _ptr(out),
                                                wsarr, _stream(stream)))


def tpi_shards_layer_prefill(cfg, weights: Sequence[tpi_layer_weights], kvs: Optional[Sequence[tpi_kv_layer]],
                             pos0: int, n_tokens: int, phase: int, h_in, partial_outs, workspaces, stream=None) -> None:
    n = len(weights)
    warr = weights if isinstance(weights, C.Array) else (tpi_layer_weights * n)(*weights)
    if kvs is None:
        karr = None
    else:
        karr = kvs if isinstance(kvs, C.Array) else (tpi_kv_layer * n)(*kvs)
    parr = partial_outs if isinstance(partial_outs, C.Array) else (C.c_void_p * n)(*[_ptr(p) for p in partial_outs])
    wsarr = workspaces if isinstance(workspaces, C.Array) else (C.c_void_p * n)(*[_ptr(p) for p in workspaces])
    _check(lib().tpi_shards_layer_prefill(C.byref(cfg), n, warr, karr, pos0, n_tokens, phase, _ptr(h_in), parr,
                                          wsarr, _stream(stream)))


def tpi_shard_layer_prefill(cfg, weights: tpi_layer_weights, kv: Optional[tpi_kv_layer], pos0: int,
                            n_tokens: int, phase: int, h_in, partial_out, workspace, stream=None) -> None:
    _check(lib().tpi_shard_layer_prefill(C.byref(cfg), C.byref(weights),
                                         C.byref(kv) if kv is not None else None, pos0, n_tokens,
                                         phase, _ptr(h_in), _ptr(partial_out), _ptr(workspace),
                                         _stream(stream)))


def tpi_star_reduce(partials, residual, out, length: Optional[int] = None, stream=None) -> None:
    """partials: sequence of tensors / addresses (rank order) or a prepared
    ``(c_void_p * n)`` array; length defaults to out.numel()."""
    if isinstance(partials, C.Array):
        arr, n = partials, len(partials)
    else:
        n = len(partials)
        arr = (C.c_void_p * max(n, 1))(*[_ptr(p) for p in partials])
    if length is None:
        length = out.numel()
    _check(lib().tpi_star_reduce(arr, n, length, _ptr(residual), _ptr(out), _stream(stream)))


def tpi_star_reduce_bf16(partials, residual, out, out_bf16, length: Optional[int] = None, stream=None) -> None:
    if isinstance(partials, C.Array):
        arr, n = partials, len(partials)
    else:
        n = len(partials)
        arr = (C.c_void_p * max(n, 1))(*[_ptr(p) for p in partials])
    if length is None:
        length = out.numel()
    _check(lib().tpi_star_reduce_bf16(arr, n, length, _ptr(residual), _ptr(out), _ptr(out_bf16), _stream(stream)))


def tpi_prof_enable(stage: int, capacity: int = 0) -> None:
    _check(lib().tpi_prof_enable(stage, capacity))


def tpi_prof_read():
    """(sum of the timed launches' durations in ms, number of launches)."""
    ms, n = C.c_double(), C.c_int32()
    _check(lib().tpi_prof_read(C.byref(ms), C.byref(n)))
    return ms.value, n.value


def tpi_decoder_workspace_bytes(cfg: tpi_shard_cfg, n_layers: int) -> int:
    return int(lib().tpi_decoder_workspace_bytes(C.byref(cfg), n_layers))


class Decoder:
    """tpi_decoder_* as an object: one device's shard, all layers of a token per launch."""

    def __init__(self, cfg, weights: Sequence[tpi_layer_weights], kvs: Sequence[tpi_kv_layer], rank: int = 0,
                 peer_attn: Optional[Sequence] = None, peer_ffn: Optional[Sequence] = None, stream=None):
        n = len(weights)
        self._h = C.c_void_p()
        nbytes = tpi_decoder_workspace_bytes(cfg, n)
        if nbytes == 0:
            raise TpiError(TPI_EINVAL, "bad shard configuration")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        warr = weights if isinstance(weights, C.Array) else (tpi_layer_weights * n)(*weights)
        karr = kvs if isinstance(kvs, C.Array) else (tpi_kv_layer * n)(*kvs)
        n_ranks = len(peer_attn) if peer_attn is not None else 1
        pa = pf = None
        if n_ranks > 1:
            pa = (C.c_void_p * n_ranks)(*[_ptr(p) if i != rank else None for i, p in enumerate(peer_attn)])
            pf = (C.c_void_p * n_ranks)(*[_ptr(p) if i != rank else None for i, p in enumerate(peer_ffn)])
        self._keep = (weights, kvs, peer_attn, peer_ffn)
        _check(lib().tpi_decoder_create(C.byref(self._h), C.byref(cfg), n, warr, karr, n_ranks, rank, pa, pf,
                                        _ptr(self.workspace), _stream(stream)))

    @property
    def grid(self) -> int:
        return int(lib().tpi_decoder_grid(self._h))

    def token(self, pos: int, h_in, h_out, stream=None) -> None:
        _check(lib().tpi_decoder_token(self._h, pos, _ptr(h_in), _ptr(h_out), _stream(stream)))

    def status(self, stream=None) -> None:
        _check(lib().tpi_decoder_status(self._h, _stream(stream)))

    def destroy(self) -> None:
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(lib().tpi_decoder_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def tpi_embed_token(w_emb, token: int, h_out, stream=None) -> None:
    """w_emb: [vocab][hidden] fp32 tensor."""
    _check(lib().tpi_embed_token(_ptr(w_emb), w_emb.shape[0], w_emb.shape[1], token, _ptr(h_out), _stream(stream)))


def tpi_lm_head(final_norm, w_head, h_in, logits, rms_eps: float = 1e-5, stream=None) -> None:
    """w_head: [vocab][hidden] fp32 tensor; logits: [vocab] fp32."""
    _check(lib().tpi_lm_head(_ptr(final_norm), _ptr(w_head), w_head.shape[0], w_head.shape[1], rms_eps, _ptr(h_in),
                             _ptr(logits), _stream(stream)))


def tpi_next_token(logits, u: float, token_out, probs=None, stream=None) -> None:
    """u < 0: largest logit; 0 <= u < 1: inverse CDF at u.  token_out: int32 device tensor of one element."""
    _check(lib().tpi_next_token(_ptr(logits), logits.numel(), u, _ptr(probs), _ptr(token_out), _stream(stream)))


class tpi_probe_result(C.Structure):
    _fields_ = [("us_total", C.c_double), ("tb_per_s", C.c_double), ("us_per_segment", C.c_double),
                ("segment_mb", C.c_double), ("spread_us", C.c_double), ("chain_us", C.c_double),
                ("segments", C.c_int32), ("results_ok", C.c_int32), ("gave_up", C.c_int32)]


class tpi_gemm_probe_result(C.Structure):
    _fields_ = [("us_per_launch", C.c_double), ("tflop_per_launch", C.c_double), ("tflops", C.c_double),
                ("result_ok", C.c_int32)]


def tpi_probe_gemm_loop(leave_out: int, reps: int = 5, stream=None) -> dict:
    l = lib()
    l.tpi_probe_gemm_loop.restype = C.c_int
    l.tpi_probe_gemm_loop.argtypes = [C.c_int32, C.c_int32, C.POINTER(tpi_gemm_probe_result), C.c_void_p]
    r = tpi_gemm_probe_result()
    _check(l.tpi_probe_gemm_loop(leave_out, reps, C.byref(r), _stream(stream)))
    return {k: getattr(r, k) for k, _ in tpi_gemm_probe_result._fields_}


def tpi_probe_handover(total_bytes: int, segment_kib_per_wave: int, mode: int, reps: int = 3, stream=None) -> dict:
    """Measurement aid: see include/tpi.h.  Returns the result structure as a dict."""
    l = lib()
    l.tpi_probe_handover.restype = C.c_int
    l.tpi_probe_handover.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.POINTER(tpi_probe_result), C.c_void_p]
    r = tpi_probe_result()
    _check(l.tpi_probe_handover(total_bytes, segment_kib_per_wave, mode, reps, C.byref(r), _stream(stream)))
    return {k: getattr(r, k) for k, _ in tpi_probe_result._fields_}


class Sim:
    """tpi_sim_*: the host model of queues, events and copies that a window can run on instead of the GPU."""

    def __init__(self, seed: int = 0):
        self._h = C.c_void_p()
        self._hashes = []          # the model writes into these when it executes the reads
        l = lib()
        l.tpi_sim_stream.restype = C.c_void_p
        l.tpi_sim_stream.argtypes = [C.c_void_p]
        l.tpi_sim_read.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_double, C.POINTER(C.c_uint64),
                                   C.POINTER(C.c_double)]
        l.tpi_sim_set_copy_rate.argtypes = [C.c_void_p, C.c_double]
        l.tpi_sim_stream_time.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
        l.tpi_sim_hash.restype = C.c_uint64
        l.tpi_sim_hash.argtypes = [C.c_void_p, C.c_size_t]
        l.tpi_sim_run.argtypes = [C.c_void_p]
        l.tpi_sim_destroy.argtypes = [C.c_void_p]
        l.tpi_sim_create.argtypes = [C.POINTER(C.c_void_p), C.c_uint64]
        _check(l.tpi_sim_create(C.byref(self._h), seed))

    def stream(self) -> int:
        return lib().tpi_sim_stream(self._h)

    def read(self, stream: int, ptr: int, nbytes: int, cost_ms: float = 0.0):
        """Queues a kernel that reads the range and takes cost_ms; returns (hash cell, start-time cell), filled
        in once the model has run it."""
        cell, start = C.c_uint64(0), C.c_double(-1.0)
        self._hashes.append((cell, start))
        _check(lib().tpi_sim_read(self._h, stream, ptr, nbytes, cost_ms, C.byref(cell), C.byref(start)))
        return cell, start

    def set_copy_rate(self, bytes_per_ms: float) -> None:
        _check(lib().tpi_sim_set_copy_rate(self._h, bytes_per_ms))

    def stream_time(self, stream: int) -> float:
        ms = C.c_double()
        _check(lib().tpi_sim_stream_time(self._h, stream, C.byref(ms)))
        return ms.value

    def run(self) -> None:
        _check(lib().tpi_sim_run(self._h))

    @staticmethod
    def hash(ptr: int, nbytes: int) -> int:
        l = lib()
        l.tpi_sim_hash.restype = C.c_uint64
        l.tpi_sim_hash.argtypes = [C.c_void_p, C.c_size_t]
        return l.tpi_sim_hash(ptr, nbytes)

    def destroy(self) -> None:
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(lib().tpi_sim_destroy(h))


class Window:
    """tpi_window_* as an object; ``slot(layer)`` mirrors the paper's
    wait_and_release context manager."""

    def __init__(self, host_blobs: Sequence[torch.Tensor], device_slots: torch.Tensor,
                 window_layers: int, layer_bytes: int):
        self._h = C.c_void_p()
        self._keep = (list(host_blobs), device_slots)
        n = len(host_blobs)
        arr = (C.c_void_p * n)(*[_ptr(b) for b in host_blobs])
        _check(lib().tpi_window_create(C.byref(self._h), n, window_layers, layer_bytes, arr,
                                       _ptr(device_slots)))

    @classmethod
    def from_blocks(cls, blocks, classes, sim: "Optional[Sim]" = None) -> "Window":
        """tpi_window_create_blocks.  blocks: sequence of (host_tensor, nbytes, slot_class, resident) with
        ``resident`` a device tensor / address for a retained block, else None; classes: sequence of
        (device_tensor, slot_bytes, n_slots).  Block indices then take the place of layer indices.
        With ``sim`` the window runs on that host model (tpi_window_create_blocks_sim): every pointer is
        then an address in host memory."""
        self = cls.__new__(cls)
        self._h = C.c_void_p()
        self._keep = (list(blocks), list(classes))
        barr = (tpi_window_block * len(blocks))()
        for i, (host, nbytes, slot_class, resident) in enumerate(blocks):
            barr[i] = tpi_window_block(_ptr(host), nbytes, slot_class, 1 if resident is not None else 0, _ptr(resident))
        carr = (tpi_window_slots * len(classes))()
        for i, (base, slot_bytes, n_slots) in enumerate(classes):
            carr[i] = tpi_window_slots(_ptr(base), slot_bytes, n_slots)
        if sim is not None:
            self._keep += (sim,)
            _check(lib().tpi_window_create_blocks_sim(C.byref(self._h), sim._h, len(blocks), barr, len(classes), carr))
        else:
            _check(lib().tpi_window_create_blocks(C.byref(self._h), len(blocks), barr, len(classes), carr))
        return self

    @classmethod
    def from_files(cls, blocks, classes, n_staging: int = 2, n_readers: int = 1, sim: "Optional[Sim]" = None) -> "Window":
        """tpi_window_create_files.  blocks: sequence of (path, offset, nbytes, slot_class, resident);
        classes as in from_blocks."""
        self = cls.__new__(cls)
        self._h = C.c_void_p()
        self._keep = (list(blocks), list(classes))
        barr = (tpi_window_file_block * len(blocks))()
        for i, (path, offset, nbytes, slot_class, resident) in enumerate(blocks):
            barr[i] = tpi_window_file_block(os.fsencode(path), offset, nbytes, slot_class,
                                            1 if resident is not None else 0, _ptr(resident))
        carr = (tpi_window_slots * len(classes))()
        for i, (base, slot_bytes, n_slots) in enumerate(classes):
            carr[i] = tpi_window_slots(_ptr(base), slot_bytes, n_slots)
        if sim is not None:
            self._keep += (sim,)
            _check(lib().tpi_window_create_files_sim(C.byref(self._h), sim._h, len(blocks), barr, len(classes), carr,
                                                     n_staging, n_readers))
        else:
            _check(lib().tpi_window_create_files(C.byref(self._h), len(blocks), barr, len(classes), carr, n_staging,
                                                 n_readers))
        return self

    def calibrate(self, stream=None) -> int:
        """tpi_window_calibrate: returns the number of copy streams tried (1: the first one was independent)."""
        l = lib()
        l.tpi_window_calibrate.restype = C.c_int
        l.tpi_window_calibrate.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
        n = C.c_int32(0)
        _check(l.tpi_window_calibrate(self._h, _stream(stream), C.byref(n)))
        return n.value

    def read_ms(self) -> float:
        ms = C.c_double()
        _check(lib().tpi_window_read_stats(self._h, C.byref(ms)))
        return ms.value

    def prefetch(self, layer: int) -> None:
        _check(lib().tpi_window_prefetch(self._h, layer))

    def acquire(self, layer: int, stream=None) -> int:
        out = C.c_void_p()
        _check(lib().tpi_window_acquire(self._h, layer, _stream(stream), C.byref(out)))
        return out.value

    def release(self, layer: int, stream=None) -> None:
        _check(lib().tpi_window_release(self._h, layer, _stream(stream)))

    def bytes_copied(self) -> int:
        """Bytes requested so far; unlike copy_stats this does not wait for the copy stream."""
        b = C.c_uint64()
        _check(lib().tpi_window_copy_stats(self._h, None, C.byref(b)))
        return b.value

    def copy_stats(self):
        ms, b = C.c_double(), C.c_uint64()
        _check(lib().tpi_window_copy_stats(self._h, C.byref(ms), C.byref(b)))
        return ms.value, b.value

    def destroy(self) -> None:
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(lib().tpi_window_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
