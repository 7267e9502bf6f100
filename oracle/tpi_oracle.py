"""TEST INFRASTRUCTURE -- not part of the product path.

ctypes front end of the plain C oracle in ``tpi_oracle.c`` (one shard's
attention block and FFN block of a Llama-style decoder layer, the fixed-order
star all-reduce sum; TPI-LLM Sec. 3.1 Step 3, Eq. 1 and Eq. 2).  Only tests,
the smoke check and the benchmark's cpu_baseline leg may import this module.
It never imports the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tpi_oracle.c")
_LIB = os.path.join(_HERE, "libtpi_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, fp64 order as written)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fno-fast-math",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q", C.c_int32), ("n_kv", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("max_seq", C.c_int32),
                ("rms_eps", C.c_double), ("rope_base", C.c_double)]


@dataclass(frozen=True)
class ShardCfg:
    """Shape of one device's shard of one decoder layer."""
    hidden: int
    n_q: int
    n_kv: int
    head_dim: int
    ffn: int
    max_seq: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    def _c(self) -> _Cfg:
        return _Cfg(self.hidden, self.n_q, self.n_kv, self.head_dim, self.ffn, self.max_seq,
                    self.rms_eps, self.rope_base)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_num_threads.restype = C.c_int
        _lib.orc_attn_block.restype = C.c_int
        _lib.orc_ffn_block.restype = C.c_int
        _lib.orc_reduce_seq_f32.restype = C.c_int
        _lib.orc_reduce_f64.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(C.c_int(n))


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def rmsnorm(x, g, eps=1e-5):
    x = _f32(x); g = _f32(g, x.shape)
    out = np.empty(x.shape[0], np.float64)
    lib().orc_rmsnorm(_p(x), _p(g), C.c_int32(x.shape[0]), C.c_double(eps), _p(out))
    return out


def matvec(W, x):
    W = _f32(W); x = np.ascontiguousarray(x, np.float64)
    assert W.ndim == 2 and x.shape == (W.shape[1],)
    y = np.empty(W.shape[0], np.float64)
    lib().orc_matvec(_p(W), C.c_int64(W.shape[0]), C.c_int64(W.shape[1]), _p(x), _p(y))
    return y


def rope(v, n_heads, d, pos, base=10000.0):
    """Rotated copy of v ([n_heads*d], fp64)."""
    out = np.array(v, dtype=np.float64, copy=True).reshape(-1)
    assert out.shape[0] == n_heads * d
    lib().orc_rope(_p(out), C.c_int32(n_heads), C.c_int32(d), C.c_int32(pos), C.c_double(base))
    return out


def attn_block(cfg: ShardCfg, g1, w_qkv, w_o, K, V, pos0, h_in, want_debug=False):
    """Attention block of one shard.  K, V: float32 [n_kv][max_seq][d], updated
    IN PLACE at slots pos0..pos0+n-1.  h_in: [h] (decode) or [n][h].
    Returns partial (fp64, same leading shape as h_in) and, with want_debug, a
    dict with q, o and the last token's softmax rows."""
    h, d = cfg.hidden, cfg.head_dim
    dq, dkv = cfg.n_q * d, cfg.n_kv * d
    h_in = _f32(h_in)
    single = h_in.ndim == 1
    x = h_in.reshape(1, h) if single else h_in
    n = x.shape[0]
    g1 = _f32(g1, (h,)); w_qkv = _f32(w_qkv, (dq + 2 * dkv, h)); w_o = _f32(w_o, (h, dq))
    for a in (K, V):
        assert a.dtype == np.float32 and a.flags.c_contiguous
        assert a.shape == (cfg.n_kv, cfg.max_seq, d), a.shape
    partial = np.empty((n, h), np.float64)
    q = o = pr = None
    if want_debug:
        q = np.empty((n, dq), np.float64); o = np.empty((n, dq), np.float64)
        pr = np.empty((cfg.n_q, pos0 + n), np.float64)
    c = cfg._c()
    rc = lib().orc_attn_block(C.byref(c), _p(g1), _p(w_qkv), _p(w_o), _p(K), _p(V),
                              C.c_int32(pos0), C.c_int32(n), _p(x), _p(partial),
                              _p(q), _p(o), _p(pr))
    if rc != 0:
        raise ValueError("orc_attn_block: bad argument")
    out = partial[0] if single else partial
    if want_debug:
        return out, {"q": q[0] if single else q, "o": o[0] if single else o, "probs": pr}
    return out


def ffn_block(cfg: ShardCfg, g2, w_gate, w_up, w_down, h_in, want_debug=False):
    """FFN block of one shard.  Returns partial (fp64)."""
    h, s = cfg.hidden, cfg.ffn
    h_in = _f32(h_in)
    single = h_in.ndim == 1
    x = h_in.reshape(1, h) if single else h_in
    n = x.shape[0]
    g2 = _f32(g2, (h,)); w_gate = _f32(w_gate, (s, h)); w_up = _f32(w_up, (s, h))
    w_down = _f32(w_down, (h, s))
    partial = np.empty((n, h), np.float64)
    act = np.empty((n, s), np.float64) if want_debug else None
    c = cfg._c()
    rc = lib().orc_ffn_block(C.byref(c), _p(g2), _p(w_gate), _p(w_up), _p(w_down),
                             C.c_int32(n), _p(x), _p(partial), _p(act))
    if rc != 0:
        raise ValueError("orc_ffn_block: bad argument")
    out = partial[0] if single else partial
    if want_debug:
        return out, {"act": act[0] if single else act}
    return out


def reduce_seq_f32(partials, residual=None):
    """fp32 sum in rank order 0..N-1, then + residual: the bit pattern the star
    all-reduce must produce."""
    ps = [_f32(p).reshape(-1) for p in partials]
    n = len(ps); ln = ps[0].shape[0]
    assert all(p.shape[0] == ln for p in ps)
    arr = (C.c_void_p * n)(*[p.ctypes.data for p in ps])
    res = _f32(residual).reshape(-1) if residual is not None else None
    out = np.empty(ln, np.float32)
    rc = lib().orc_reduce_seq_f32(arr, C.c_int32(n), C.c_int64(ln), _p(res), _p(out))
    if rc != 0:
        raise ValueError("orc_reduce_seq_f32: bad argument")
    return out.reshape(np.shape(partials[0]))


def reduce_f64(partials, residual=None):
    ps = [np.ascontiguousarray(p, np.float64).reshape(-1) for p in partials]
    n = len(ps); ln = ps[0].shape[0]
    arr = (C.c_void_p * n)(*[p.ctypes.data for p in ps])
    res = _f32(residual).reshape(-1) if residual is not None else None
    out = np.empty(ln, np.float64)
    rc = lib().orc_reduce_f64(arr, C.c_int32(n), C.c_int64(ln), _p(res), _p(out))
    if rc != 0:
        raise ValueError("orc_reduce_f64: bad argument")
    return out.reshape(np.shape(partials[0]))


def layer_decode(cfg: ShardCfg, shards, kv, pos, h_in):
    """One decoder layer over N emulated shards, one token (Alg. 1, loop body):
    attention partials -> reduce + shortcut -> FFN partials -> reduce + shortcut.
    shards: list of dicts (attn_norm, w_qkv, w_o, ffn_norm, w_gate, w_up, w_down);
    kv: list of (K, V) per shard, updated in place.  Interface values (partials,
    H_attn, H_ffn) are fp32.  Returns (H_ffn, H_attn, attn_partials, ffn_partials)."""
    h_in = _f32(h_in)
    pa = [attn_block(cfg, s["attn_norm"], s["w_qkv"], s["w_o"], kv[r][0], kv[r][1], pos, h_in)
          .astype(np.float32) for r, s in enumerate(shards)]
    h_attn = reduce_seq_f32(pa, h_in)
    pf = [ffn_block(cfg, s["ffn_norm"], s["w_gate"], s["w_up"], s["w_down"], h_attn)
          .astype(np.float32) for s in shards]
    h_ffn = reduce_seq_f32(pf, h_attn)
    return h_ffn, h_attn, pa, pf


# ---------------------------------------------------------------------------
# The ends of the token loop, master only (Alg. 1 "Preprocess" and "Postprocess"; Sec. 3.1 Step 4:
# the summed output passes the final norm and the task head, softmax gives the distribution of the
# next token, which is then sampled).
# ---------------------------------------------------------------------------

def embed_token(w_emb, token):
    """Input embedding of one token index: row `token` of W_emb [vocab][h]."""
    w_emb = np.asarray(w_emb)
    if not 0 <= token < w_emb.shape[0]:
        raise ValueError("token outside the vocabulary")
    return np.array(w_emb[token], dtype=np.float32, copy=True)


def lm_head(final_norm, w_head, h_in, eps=1e-5):
    """logits[v] = W_head[v] . rmsnorm(h_in) (fp64)."""
    return matvec(w_head, rmsnorm(h_in, final_norm, eps))


def softmax(logits):
    z = np.asarray(logits, np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def greedy_token(logits):
    """Index of the largest logit, the lowest index among equals."""
    z = np.asarray(logits)
    best = 0
    for i in range(1, z.shape[0]):
        if z[i] > z[best]:
            best = i
    return best


def sample_token(logits, u):
    """Inverse-CDF sampling with a uniform draw u in [0, 1) supplied by the caller: the first index whose
    cumulative probability exceeds u (the last index if rounding leaves the total below u)."""
    p = softmax(logits)
    acc = 0.0
    for i in range(p.shape[0]):
        acc += p[i]
        if acc > u:
            return i
    return p.shape[0] - 1

