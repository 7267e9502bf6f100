"""Seeded synthetic inputs shared by the tests, the smoke check and the
benchmark.  This module draws random numbers and lays tensors out; it holds
none of the method's arithmetic and imports neither the oracle nor the HIP
binding.

Recipe: weight matrices ~ N(0, 0.02^2); RMSNorm gains 1 + N(0, 0.02^2);
hidden state and pre-filled KV-cache slots ~ N(0, 1).  Draw order is fixed:
layer -> shard -> (attn_norm, w_qkv, w_o, ffn_norm, w_gate, w_up, w_down), then
the caches layer -> shard -> (K, V), then the hidden state.
"""
from __future__ import annotations

import numpy as np

WEIGHT_STD = 0.02
TENSOR_ORDER = ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate", "w_up", "w_down")


def shard_tensor_shapes(hidden, nq, nkv, d, ffn_local):
    """Shapes of one layer-shard's tensors, in blob order."""
    return {
        "attn_norm": (hidden,),
        "w_qkv": ((nq + 2 * nkv) * d, hidden),   # rows: Q heads, K heads, V heads
        "w_o": (hidden, nq * d),
        "ffn_norm": (hidden,),
        "w_gate": (ffn_local, hidden),
        "w_up": (ffn_local, hidden),
        "w_down": (hidden, ffn_local),
    }


def make_layer_shard(rng: np.random.Generator, hidden, nq, nkv, d, ffn_local):
    """One layer-shard's weights as float32 numpy arrays."""
    out = {}
    for name, shape in shard_tensor_shapes(hidden, nq, nkv, d, ffn_local).items():
        x = rng.standard_normal(shape, dtype=np.float32) * np.float32(WEIGHT_STD)
        if name.endswith("_norm"):
            x = np.float32(1.0) + x
        out[name] = x
    return out


def make_stack(seed, n_layers, n_shards, hidden, nq, nkv, d, ffn_local, max_seq, n_cached):
    """Weights [layer][shard], KV caches [layer][shard] = (K, V) float32
    [nkv][max_seq][d] with slots 0..n_cached-1 ~ N(0,1) and the rest zero, and
    the input hidden state [hidden]."""
    rng = np.random.default_rng(seed)
    weights = [[make_layer_shard(rng, hidden, nq, nkv, d, ffn_local) for _ in range(n_shards)]
               for _ in range(n_layers)]
    caches = []
    for _ in range(n_layers):
        row = []
        for _ in range(n_shards):
            K = np.zeros((nkv, max_seq, d), np.float32)
            V = np.zeros((nkv, max_seq, d), np.float32)
            K[:, :n_cached] = rng.standard_normal((nkv, n_cached, d), dtype=np.float32)
            V[:, :n_cached] = rng.standard_normal((nkv, n_cached, d), dtype=np.float32)
            row.append((K, V))
        caches.append(row)
    h_in = rng.standard_normal(hidden, dtype=np.float32)
    return weights, caches, h_in


def stack_from_shape(shape, seed=0, max_seq=None, n_cached=16, n_layers=None):
    """make_stack for a configs.ModelShape."""
    L = shape.n_layers if n_layers is None else n_layers
    ms = max_seq if max_seq is not None else n_cached + 8
    return make_stack(seed, L, shape.n_shards, shape.hidden, shape.nq_local, shape.nkv_local,
                      shape.head_dim, shape.ffn_local, ms, n_cached)


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), returned as
    float32: the value set a bf16 tensor can hold."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def blob_layout_bytes(hidden, nq, nkv, d, ffn_local, matrix_itemsize):
    """Byte layout of one contiguous layer-shard blob: the tensors of TENSOR_ORDER, each starting on a
    256-byte boundary; norm gains are fp32, matrices have `matrix_itemsize` bytes per element (4: fp32
    decode weights, 2: bf16 prefill weights).  Returns ({name: (byte_offset, shape, itemsize)}, total_bytes)."""
    shapes = shard_tensor_shapes(hidden, nq, nkv, d, ffn_local)
    off, out = 0, {}
    for name in TENSOR_ORDER:
        item = 4 if name.endswith("_norm") else matrix_itemsize
        out[name] = (off, shapes[name], item)
        off += (int(np.prod(shapes[name])) * item + 255) // 256 * 256
    return out, off

