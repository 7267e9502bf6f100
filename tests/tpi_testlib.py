"""Helpers for the GPU parity tests: move a synthetic stack to the device, run
the HIP path through the C ABI, run the oracle on the same arrays."""
from __future__ import annotations

import numpy as np
import torch

from oracle import tpi_oracle as O
from paper_2410_00531_amd import binding as B
from paper_2410_00531_amd import synth

FP32_TOL = 1e-4      # max |gpu - oracle| / max |oracle|, fp32 paths
BF16_TOL = 2e-2      # bf16 prefill


def rel_err(got, ref) -> float:
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


class GpuShard:
    """One layer-shard on the device: weights, KV cache, output and workspace."""

    def __init__(self, cfg: B.tpi_shard_cfg, w_np: dict, K_np, V_np, dev="cuda:0"):
        self.cfg = cfg
        self.w = {k: torch.from_numpy(np.ascontiguousarray(v)).to(dev) for k, v in w_np.items()}
        self.K = torch.from_numpy(K_np.copy()).to(dev)
        self.V = torch.from_numpy(V_np.copy()).to(dev)
        self.weights = B.make_weights(self.w)
        self.kv = B.make_kv(self.K, self.V)
        self.partial = torch.empty(cfg.hidden, dtype=torch.float32, device=dev)
        nbytes = B.tpi_workspace_bytes(cfg, 1)
        assert nbytes > 0
        # poison the workspace: it must need no initialisation
        self.ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device=dev)


def ocfg(cfg: B.tpi_shard_cfg) -> O.ShardCfg:
    return O.ShardCfg(cfg.hidden, cfg.n_q_local, cfg.n_kv_local, cfg.head_dim, cfg.ffn_local,
                      cfg.max_seq, float(cfg.rms_eps), float(cfg.rope_base))


def random_shard_np(rng, cfg: B.tpi_shard_cfg, n_cached: int, kv_scale=1.0):
    w = synth.make_layer_shard(rng, cfg.hidden, cfg.n_q_local, cfg.n_kv_local, cfg.head_dim,
                               cfg.ffn_local)
    K = np.zeros((cfg.n_kv_local, cfg.max_seq, cfg.head_dim), np.float32)
    V = np.zeros_like(K)
    if n_cached:
        K[:, :n_cached] = rng.standard_normal((cfg.n_kv_local, n_cached, cfg.head_dim), dtype=np.float32) * kv_scale
        V[:, :n_cached] = rng.standard_normal((cfg.n_kv_local, n_cached, cfg.head_dim), dtype=np.float32)
    return w, K, V


def check_attn_phase(cfg, w, K, V, pos, h_in, tol=FP32_TOL, sentinel=True):
    """Runs the attention phase on GPU and oracle from the same arrays; checks
    the partial, the cache values at slot pos, and that no other slot changed
    (bit-exact).  Returns (gpu partial, oracle partial)."""
    K = K.copy(); V = V.copy()
    if sentinel:
        pat = np.frombuffer(np.uint32(0x7FC0BEEF).tobytes(), np.float32)[0]
        K[:, pos:] = pat; V[:, pos:] = pat
    sh = GpuShard(cfg, w, K, V)
    x = torch.from_numpy(h_in).cuda()
    B.tpi_shard_layer_decode(cfg, sh.weights, sh.kv, pos, B.TPI_PHASE_ATTN, x, sh.partial, sh.ws)
    torch.cuda.synchronize()
    Kg, Vg = sh.K.cpu().numpy(), sh.V.cpu().numpy()
    Ko, Vo = K.copy(), V.copy()
    ref = O.attn_block(ocfg(cfg), w["attn_norm"], w["w_qkv"], w["w_o"], Ko, Vo, pos, h_in)
    got = sh.partial.cpu().numpy()
    # slot indexing: exactly slot pos of every local KV head changed
    for g_arr, before in ((Kg, K), (Vg, V)):
        changed = (g_arr.view(np.uint32) != before.view(np.uint32)).any(axis=2)
        expect = np.zeros_like(changed); expect[:, pos] = True
        assert np.array_equal(changed, expect), "cache slots other than pos were touched (or pos was not)"
    assert rel_err(Kg[:, pos], Ko[:, pos]) <= tol
    assert rel_err(Vg[:, pos], Vo[:, pos]) <= tol
    e = rel_err(got, ref)
    assert e <= tol, f"attention partial rel err {e:.3e}"
    return got, ref


def check_ffn_phase(cfg, w, h_in, tol=FP32_TOL):
    sh = GpuShard(cfg, w, np.zeros((cfg.n_kv_local, cfg.max_seq, cfg.head_dim), np.float32),
                  np.zeros((cfg.n_kv_local, cfg.max_seq, cfg.head_dim), np.float32))
    x = torch.from_numpy(h_in).cuda()
    B.tpi_shard_layer_decode(cfg, sh.weights, None, 0, B.TPI_PHASE_FFN, x, sh.partial, sh.ws)
    torch.cuda.synchronize()
    ref = O.ffn_block(ocfg(cfg), w["ffn_norm"], w["w_gate"], w["w_up"], w["w_down"], h_in)
    got = sh.partial.cpu().numpy()
    e = rel_err(got, ref)
    assert e <= tol, f"FFN partial rel err {e:.3e}"
    return got, ref


def gpu_layer_decode(cfg, shards, pos, h_in_t, h_attn_t, h_out_t, batched=True):
    """One layer over the emulated shards on the device (Alg. 1 loop body)."""
    n = len(shards)
    ws = [s.weights for s in shards]; kvs = [s.kv for s in shards]
    pouts = [s.partial for s in shards]; wss = [s.ws for s in shards]
    if batched:
        B.tpi_shards_layer_decode(cfg, ws, kvs, pos, B.TPI_PHASE_ATTN, h_in_t, pouts, wss)
    else:
        for s in shards:
            B.tpi_shard_layer_decode(cfg, s.weights, s.kv, pos, B.TPI_PHASE_ATTN, h_in_t, s.partial, s.ws)
    B.tpi_star_reduce(pouts, h_in_t, h_attn_t)
    if batched:
        B.tpi_shards_layer_decode(cfg, ws, None, pos, B.TPI_PHASE_FFN, h_attn_t, pouts, wss)
    else:
        for s in shards:
            B.tpi_shard_layer_decode(cfg, s.weights, None, pos, B.TPI_PHASE_FFN, h_attn_t, s.partial, s.ws)
    B.tpi_star_reduce(pouts, h_attn_t, h_out_t)
