"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- an unsharded layer built from PyTorch CPU library ops, a
brute-force einsum, closed forms and invariants.  No GPU involved."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import tpi_oracle as O

torch.set_num_threads(4)


# ----------------------------------------------------------------------------
# An unsharded decoder layer from library ops only (fp64), written with a
# different formulation than the oracle: complex multiplication for the rotary
# embedding, scaled_dot_product_attention for the softmax, F.linear for GEMVs.
# ----------------------------------------------------------------------------

def _rope_complex(x, pos, base):
    """x: [heads][d] fp64 tensor.  Pair (i, i+d/2) as a complex number times
    exp(i * pos * base^(-2i/d))."""
    d = x.shape[-1]
    half = d // 2
    z = torch.complex(x[..., :half], x[..., half:])
    theta = torch.tensor([base ** (-2.0 * i / d) for i in range(half)], dtype=torch.float64)
    rot = torch.polar(torch.ones(half, dtype=torch.float64), pos * theta)
    z = z * rot
    return torch.cat([z.real, z.imag], dim=-1)


def dense_layer_torch(x, full, Kc, Vc, pos, a, b, d, eps=1e-5, base=10000.0):
    """Unsharded layer: returns (H_attn, H_ffn); Kc, Vc [b][max_seq][d] fp32
    tensors updated in place at slot pos."""
    t = lambda v: torch.as_tensor(np.asarray(v), dtype=torch.float64)
    x = t(x)
    rms = lambda v, g: v * torch.rsqrt(v.pow(2).mean() + eps) * t(g)
    xn = rms(x, full["attn_norm"])
    q = F.linear(xn, t(full["w_q"])).view(a, d)
    k = F.linear(xn, t(full["w_k"])).view(b, d)
    v = F.linear(xn, t(full["w_v"])).view(b, d)
    q = _rope_complex(q, pos, base)
    k = _rope_complex(k, pos, base)
    Kc[:, pos] = k.to(torch.float32)
    Vc[:, pos] = v.to(torch.float32)
    Kf = Kc[:, :pos + 1].to(torch.float64).repeat_interleave(a // b, dim=0)   # [a][T][d]
    Vf = Vc[:, :pos + 1].to(torch.float64).repeat_interleave(a // b, dim=0)
    o = F.scaled_dot_product_attention(q.view(1, a, 1, d), Kf.view(1, a, pos + 1, d),
                                       Vf.view(1, a, pos + 1, d)).view(a * d)
    h_attn = F.linear(o, t(full["w_o"])) + x
    xn2 = rms(h_attn, full["ffn_norm"])
    act = F.silu(F.linear(xn2, t(full["w_gate"]))) * F.linear(xn2, t(full["w_up"]))
    h_ffn = F.linear(act, t(full["w_down"])) + h_attn
    return h_attn.numpy(), h_ffn.numpy()


def make_full_layer(rng, h, a, b, d, s):
    w = lambda *shape: (rng.standard_normal(shape) * 0.02).astype(np.float32)
    g = lambda: (1.0 + rng.standard_normal(h) * 0.02).astype(np.float32)
    return {"attn_norm": g(), "w_q": w(a * d, h), "w_k": w(b * d, h), "w_v": w(b * d, h),
            "w_o": w(h, a * d), "ffn_norm": g(), "w_gate": w(s, h), "w_up": w(s, h),
            "w_down": w(h, s)}


def slice_shard(full, r, N, a, b, d, s):
    """Shard r of N: q heads [r a/N, (r+1) a/N), kv heads likewise, FFN columns
    [r s/N, (r+1) s/N)  (Sec. 3.1 Step 1: split by heads and FFN columns)."""
    nq, nkv, sl = a // N, b // N, s // N
    qs = slice(r * nq * d, (r + 1) * nq * d)
    ks = slice(r * nkv * d, (r + 1) * nkv * d)
    fs = slice(r * sl, (r + 1) * sl)
    return {"attn_norm": full["attn_norm"],
            "w_qkv": np.concatenate([full["w_q"][qs], full["w_k"][ks], full["w_v"][ks]], 0),
            "w_o": np.ascontiguousarray(full["w_o"][:, qs]),
            "ffn_norm": full["ffn_norm"],
            "w_gate": full["w_gate"][fs], "w_up": full["w_up"][fs],
            "w_down": np.ascontiguousarray(full["w_down"][:, fs])}


@pytest.mark.parametrize("N", [1, 2, 4, 8])
@pytest.mark.parametrize("a,b", [(8, 8), (16, 8), (32, 8)])
def test_tp_identity_against_unsharded_torch_layer(N, a, b):
    """Sum of the N shard partials + shortcut == the unsharded layer (the
    paper's claim that the generated sequence equals single-server inference)."""
    rng = np.random.default_rng(100 + N + a)
    h, d, s, T, max_seq = 96, 16, 160, 9, 12
    full = make_full_layer(rng, h, a, b, d, s)
    x = rng.standard_normal(h).astype(np.float32)
    Kfull = np.zeros((b, max_seq, d), np.float32); Vfull = np.zeros_like(Kfull)
    Kfull[:, :T] = rng.standard_normal((b, T, d)); Vfull[:, :T] = rng.standard_normal((b, T, d))
    Kt, Vt = torch.tensor(Kfull.copy()), torch.tensor(Vfull.copy())
    ref_attn, ref_ffn = dense_layer_torch(x, full, Kt, Vt, T, a, b, d)

    cfg = O.ShardCfg(h, a // N, b // N, d, s // N, max_seq)
    nkv = b // N
    pa, caches = [], []
    for r in range(N):
        sh = slice_shard(full, r, N, a, b, d, s)
        K = np.ascontiguousarray(Kfull[r * nkv:(r + 1) * nkv]); V = np.ascontiguousarray(Vfull[r * nkv:(r + 1) * nkv])
        pa.append(O.attn_block(cfg, sh["attn_norm"], sh["w_qkv"], sh["w_o"], K, V, T, x))
        caches.append((K, V))
    h_attn = O.reduce_f64(pa, x)
    np.testing.assert_allclose(h_attn, ref_attn, rtol=0, atol=1e-12 * np.abs(ref_attn).max() + 1e-14)
    # the distributed cache, concatenated over shards, is the unsharded cache
    np.testing.assert_array_equal(np.concatenate([c[0] for c in caches], 0), Kt.numpy())
    np.testing.assert_array_equal(np.concatenate([c[1] for c in caches], 0), Vt.numpy())

    # FFN on the unsharded H_attn (fp64 values are not representable as fp32
    # inputs, so feed both sides the fp32-rounded H_attn)
    h_attn32 = ref_attn.astype(np.float32)
    t = lambda v: torch.as_tensor(np.asarray(v), dtype=torch.float64)
    xn2 = t(h_attn32) * torch.rsqrt(t(h_attn32).pow(2).mean() + 1e-5) * t(full["ffn_norm"])
    ref = (F.linear(F.silu(F.linear(xn2, t(full["w_gate"]))) * F.linear(xn2, t(full["w_up"])),
                    t(full["w_down"])) + t(h_attn32)).numpy()
    pf = [O.ffn_block(cfg, *(slice_shard(full, r, N, a, b, d, s)[k] for k in
                             ("ffn_norm", "w_gate", "w_up", "w_down")), h_attn32) for r in range(N)]
    got = O.reduce_f64(pf, h_attn32)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12 * np.abs(ref).max() + 1e-14)


def slice_uneven_shard(full, q0, q1, k0, k1, f0, f1, d):
    """A shard that owns query heads [q0, q1), KV heads [k0, k1) and FFN columns [f0, f1): the split by
    unequal proportions p_i of Sec. 3.1."""
    qs, ks, fs = slice(q0 * d, q1 * d), slice(k0 * d, k1 * d), slice(f0, f1)
    return {"attn_norm": full["attn_norm"],
            "w_qkv": np.concatenate([full["w_q"][qs], full["w_k"][ks], full["w_v"][ks]], 0),
            "w_o": np.ascontiguousarray(full["w_o"][:, qs]),
            "ffn_norm": full["ffn_norm"],
            "w_gate": full["w_gate"][fs], "w_up": full["w_up"][fs],
            "w_down": np.ascontiguousarray(full["w_down"][:, fs])}


# heads per shard (query, KV) and FFN columns per shard: proportions 1/2, 1/4, 1/4 and a ragged FFN split
UNEVEN_SPLIT = dict(a=8, b=4, d=16, s=160, q=(4, 2, 2), kv=(2, 1, 1), f=(70, 50, 40))


def test_tp_identity_with_uneven_shares():
    """Devices may hold unequal proportions p_i of the heads and FFN columns (Sec. 3.1); the sum of the
    shard partials is still the unsharded layer."""
    u = UNEVEN_SPLIT
    a, b, d, s = u["a"], u["b"], u["d"], u["s"]
    rng = np.random.default_rng(4242)
    h, T, max_seq = 96, 7, 10
    full = make_full_layer(rng, h, a, b, d, s)
    x = rng.standard_normal(h).astype(np.float32)
    Kfull = np.zeros((b, max_seq, d), np.float32); Vfull = np.zeros_like(Kfull)
    Kfull[:, :T] = rng.standard_normal((b, T, d)); Vfull[:, :T] = rng.standard_normal((b, T, d))
    Kt, Vt = torch.tensor(Kfull.copy()), torch.tensor(Vfull.copy())
    ref_attn, ref_ffn = dense_layer_torch(x, full, Kt, Vt, T, a, b, d)
    pa, shards, cfgs = [], [], []
    q0 = k0 = f0 = 0
    for nq, nkv, sl in zip(u["q"], u["kv"], u["f"]):
        sh = slice_uneven_shard(full, q0, q0 + nq, k0, k0 + nkv, f0, f0 + sl, d)
        cfg = O.ShardCfg(h, nq, nkv, d, sl, max_seq)
        K = np.ascontiguousarray(Kfull[k0:k0 + nkv]); V = np.ascontiguousarray(Vfull[k0:k0 + nkv])
        pa.append(O.attn_block(cfg, sh["attn_norm"], sh["w_qkv"], sh["w_o"], K, V, T, x))
        shards.append(sh); cfgs.append(cfg)
        q0 += nq; k0 += nkv; f0 += sl
    assert (q0, k0, f0) == (a, b, s)
    h_attn = O.reduce_f64(pa, x)
    np.testing.assert_allclose(h_attn, ref_attn, rtol=0, atol=1e-12 * np.abs(ref_attn).max() + 1e-14)
    h_attn32 = ref_attn.astype(np.float32)
    t = lambda v: torch.as_tensor(np.asarray(v), dtype=torch.float64)
    xn2 = t(h_attn32) * torch.rsqrt(t(h_attn32).pow(2).mean() + 1e-5) * t(full["ffn_norm"])
    ref = (F.linear(F.silu(F.linear(xn2, t(full["w_gate"]))) * F.linear(xn2, t(full["w_up"])),
                    t(full["w_down"])) + t(h_attn32)).numpy()
    pf = [O.ffn_block(c, sh["ffn_norm"], sh["w_gate"], sh["w_up"], sh["w_down"], h_attn32)
          for c, sh in zip(cfgs, shards)]
    np.testing.assert_allclose(O.reduce_f64(pf, h_attn32), ref, rtol=0, atol=1e-12 * np.abs(ref).max() + 1e-14)


def test_brute_force_hand_sized_case():
    """h = 4, one head per shard, d = 2, 4 FFN columns per shard, N = 2:
    every step written as an einsum over explicit index expressions."""
    rng = np.random.default_rng(7)
    h, d, sl, N, T = 4, 2, 4, 2, 3
    cfg = O.ShardCfg(h, 1, 1, d, sl, T + 1, rms_eps=1e-5, rope_base=10000.0)
    x = rng.standard_normal(h).astype(np.float32)
    tot_attn = np.zeros(h); shards = []
    for r in range(N):
        g1 = (1 + 0.1 * rng.standard_normal(h)).astype(np.float32)
        wqkv = rng.standard_normal((3 * d, h)).astype(np.float32)
        wo = rng.standard_normal((h, d)).astype(np.float32)
        K = np.zeros((1, T + 1, d), np.float32); V = np.zeros_like(K)
        K[0, :T] = rng.standard_normal((T, d)); V[0, :T] = rng.standard_normal((T, d))
        K0, V0 = K.copy(), V.copy()
        got = O.attn_block(cfg, g1, wqkv, wo, K, V, T, x)
        # brute force
        xd = x.astype(np.float64)
        xn = xd / math.sqrt((xd ** 2).sum() / h + 1e-5) * g1
        qkv = np.einsum("oi,i->o", wqkv.astype(np.float64), xn)
        ang = float(T) * 1.0            # d = 2: one pair, theta_0 = 1, angle = pos radians
        R = np.array([[math.cos(ang), -math.sin(ang)], [math.sin(ang), math.cos(ang)]])
        q = R @ qkv[0:2]; k = R @ qkv[2:4]; v = qkv[4:6]
        Kb = np.concatenate([K0[0, :T].astype(np.float64), k.astype(np.float32)[None].astype(np.float64)])
        Vb = np.concatenate([V0[0, :T].astype(np.float64), v.astype(np.float32)[None].astype(np.float64)])
        sc = np.einsum("e,te->t", q, Kb) / math.sqrt(d)
        p = np.exp(sc - sc.max()); p /= p.sum()
        o = np.einsum("t,te->e", p, Vb)
        ref = np.einsum("oe,e->o", wo.astype(np.float64), o)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)
        assert np.array_equal(K[0, T], k.astype(np.float32)) and np.array_equal(V[0, T], v.astype(np.float32))
        tot_attn += ref
    h_attn = (tot_attn + x).astype(np.float32)
    tot = np.zeros(h)
    for r in range(N):
        g2 = (1 + 0.1 * rng.standard_normal(h)).astype(np.float32)
        wg, wu = rng.standard_normal((sl, h)).astype(np.float32), rng.standard_normal((sl, h)).astype(np.float32)
        wd = rng.standard_normal((h, sl)).astype(np.float32)
        got = O.ffn_block(cfg, g2, wg, wu, wd, h_attn)
        xd = h_attn.astype(np.float64)
        xn = xd / math.sqrt((xd ** 2).sum() / h + 1e-5) * g2
        gt = np.einsum("jh,h->j", wg.astype(np.float64), xn); up = np.einsum("jh,h->j", wu.astype(np.float64), xn)
        ref = np.einsum("hj,j->h", wd.astype(np.float64), gt / (1 + np.exp(-gt)) * up)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------
# RMSNorm
# ----------------------------------------------------------------------------

def test_rmsnorm_closed_forms():
    h, eps = 64, 1e-5
    c = 3.0
    out = O.rmsnorm(np.full(h, c, np.float32), np.ones(h, np.float32), eps)
    np.testing.assert_allclose(out, c / math.sqrt(c * c + eps), rtol=1e-14)
    rng = np.random.default_rng(1)
    x = rng.standard_normal(h).astype(np.float32)
    out = O.rmsnorm(x, np.ones(h, np.float32), eps)
    ms = float((x.astype(np.float64) ** 2).mean())
    np.testing.assert_allclose((out ** 2).mean(), ms / (ms + eps), rtol=1e-13)
    # scale invariance (eps is negligible against ms * 2^20): exact power-of-two scaling
    out2 = O.rmsnorm((x * 1024).astype(np.float32), np.ones(h, np.float32), eps)
    np.testing.assert_allclose(out2, out, rtol=1e-5)
    # gain multiplies last and elementwise; no mean subtraction (a constant offset survives)
    g = rng.standard_normal(h).astype(np.float32)
    np.testing.assert_allclose(O.rmsnorm(x, g, eps), out * g, rtol=1e-14)
    assert abs(O.rmsnorm(x + 5, np.ones(h, np.float32), eps).mean()) > 0.5


# ----------------------------------------------------------------------------
# Rotary embedding
# ----------------------------------------------------------------------------

def test_rope_position_zero_is_identity_bitwise():
    rng = np.random.default_rng(2)
    v = rng.standard_normal(3 * 64)
    out = O.rope(v, 3, 64, 0)
    assert np.array_equal(out.view(np.uint64), v.view(np.uint64))


def test_rope_d2_is_plane_rotation_by_pos_radians():
    v = np.array([1.0, 0.0])
    for pos in (1, 2, 7):
        out = O.rope(v, 1, 2, pos)
        np.testing.assert_allclose(out, [math.cos(pos), math.sin(pos)], atol=1e-15)
    out = O.rope(np.array([0.0, 1.0]), 1, 2, 1)
    np.testing.assert_allclose(out, [-math.sin(1), math.cos(1)], atol=1e-15)


def test_rope_pair_norms_and_relative_position_property():
    rng = np.random.default_rng(3)
    d = 32
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    for pos in (1, 5, 1000):
        out = O.rope(q, 1, d, pos)
        np.testing.assert_allclose(out[:d // 2] ** 2 + out[d // 2:] ** 2,
                                   q[:d // 2] ** 2 + q[d // 2:] ** 2, rtol=1e-12)
    dots = [O.rope(q, 1, d, m) @ O.rope(k, 1, d, n) for m, n in ((5, 2), (13, 10), (103, 100))]
    np.testing.assert_allclose(dots, dots[0], rtol=1e-10)
    assert abs(O.rope(q, 1, d, 5) @ O.rope(k, 1, d, 3) - dots[0]) > 1e-6
    # frequencies: pair i turns by pos * base^(-2i/d); check the slowest pair explicitly
    e = np.zeros(d); e[d // 2 - 1] = 1.0
    out = O.rope(e, 1, d, 1, base=10000.0)
    th = 10000.0 ** (-(d - 2) / d)
    np.testing.assert_allclose([out[d // 2 - 1], out[d - 1]], [math.cos(th), math.sin(th)], atol=1e-15)
    # heads are rotated independently and identically
    two = O.rope(np.concatenate([q, k]), 2, d, 9)
    np.testing.assert_array_equal(two[:d], O.rope(q, 1, d, 9))
    np.testing.assert_array_equal(two[d:], O.rope(k, 1, d, 9))


# ----------------------------------------------------------------------------
# Attention
# ----------------------------------------------------------------------------

def _rand_attn(rng, h=48, nq=4, nkv=2, d=8, T=6, max_seq=8):
    cfg = O.ShardCfg(h, nq, nkv, d, 16, max_seq)
    g1 = (1 + 0.02 * rng.standard_normal(h)).astype(np.float32)
    wqkv = (0.3 * rng.standard_normal(((nq + 2 * nkv) * d, h))).astype(np.float32)
    wo = (0.3 * rng.standard_normal((h, nq * d))).astype(np.float32)
    K = np.zeros((nkv, max_seq, d), np.float32); V = np.zeros_like(K)
    K[:, :T] = rng.standard_normal((nkv, T, d)); V[:, :T] = rng.standard_normal((nkv, T, d))
    x = rng.standard_normal(h).astype(np.float32)
    return cfg, g1, wqkv, wo, K, V, x


def test_softmax_rows_sum_to_one_and_scores_scale():
    rng = np.random.default_rng(4)
    cfg, g1, wqkv, wo, K, V, x = _rand_attn(rng)
    _, dbg = O.attn_block(cfg, g1, wqkv, wo, K, V, 6, x, want_debug=True)
    pr = dbg["probs"]
    assert pr.shape == (4, 7)
    np.testing.assert_allclose(pr.sum(1), 1.0, rtol=1e-14)
    assert (pr > 0).all()
    # ratio of two probabilities = exp((q.k_s - q.k_t)/sqrt(d)): pins the 1/sqrt(d) scale
    q = dbg["q"].reshape(4, 8)
    for j in range(4):
        g = j // 2
        lhs = math.log(pr[j, 1] / pr[j, 4])
        rhs = (q[j] @ K[g, 1].astype(np.float64) - q[j] @ K[g, 4].astype(np.float64)) / math.sqrt(8)
        assert abs(lhs - rhs) < 1e-12


def test_empty_cache_output_is_own_value():
    """pos = 0: one key, probability 1, head output == this token's V."""
    rng = np.random.default_rng(5)
    cfg, g1, wqkv, wo, K, V, x = _rand_attn(rng, T=0)
    _, dbg = O.attn_block(cfg, g1, wqkv, wo, K, V, 0, x, want_debug=True)
    o = dbg["o"].reshape(4, 8)
    for j in range(4):
        np.testing.assert_array_equal(o[j], V[j // 2, 0].astype(np.float64))


def test_equal_keys_give_mean_of_values_and_slot_permutation_invariance():
    rng = np.random.default_rng(6)
    cfg, g1, wqkv, wo, K, V, x = _rand_attn(rng)
    # W_K = 0 -> the new key is 0; make all cached keys 0 as well -> uniform softmax
    wq0 = wqkv.copy(); wq0[4 * 8:4 * 8 + 2 * 8] = 0
    K0 = np.zeros_like(K)
    V1 = V.copy()
    _, dbg = O.attn_block(cfg, g1, wq0, wo, K0, V1, 6, x, want_debug=True)
    o = dbg["o"].reshape(4, 8)
    for j in range(4):
        np.testing.assert_allclose(o[j], V1[j // 2, :7].astype(np.float64).mean(0), rtol=1e-13, atol=1e-15)
    # permuting cached slots (K and V together) leaves the output unchanged
    perm = rng.permutation(6)
    Ka, Va = K.copy(), V.copy()
    Kb, Vb = K.copy(), V.copy(); Kb[:, :6] = K[:, perm]; Vb[:, :6] = V[:, perm]
    pa = O.attn_block(cfg, g1, wqkv, wo, Ka, Va, 6, x)
    pb = O.attn_block(cfg, g1, wqkv, wo, Kb, Vb, 6, x)
    np.testing.assert_allclose(pa, pb, rtol=1e-12, atol=1e-14)


def test_gqa_equals_mha_with_repeated_kv_heads():
    """nq = 4, nkv = 2 equals nq = nkv = 4 with each KV head's projection and
    cache repeated for the two query heads of its group."""
    rng = np.random.default_rng(8)
    cfg, g1, wqkv, wo, K, V, x = _rand_attn(rng)
    d = 8
    wq, wk, wv = wqkv[:32], wqkv[32:48], wqkv[48:64]
    rep = lambda w: np.repeat(w.reshape(2, d, -1), 2, axis=0).reshape(4 * d, -1)
    wqkv_mha = np.concatenate([wq, rep(wk), rep(wv)], 0)
    cfg_mha = O.ShardCfg(cfg.hidden, 4, 4, d, cfg.ffn, cfg.max_seq)
    Km, Vm = np.repeat(K, 2, axis=0).copy(), np.repeat(V, 2, axis=0).copy()
    pa = O.attn_block(cfg, g1, wqkv, wo, K, V, 6, x)
    pb = O.attn_block(cfg_mha, g1, wqkv_mha, wo, Km, Vm, 6, x)
    np.testing.assert_allclose(pa, pb, rtol=1e-13, atol=1e-15)


def test_kv_append_touches_exactly_slot_pos():
    rng = np.random.default_rng(9)
    for pos, max_seq in ((0, 8), (5, 8), (7, 8)):
        cfg, g1, wqkv, wo, K, V, x = _rand_attn(rng, T=pos, max_seq=max_seq)
        sentinel = np.float32(np.frombuffer(np.uint32(0x7FC0BEEF).tobytes(), np.float32)[0])
        K[:, pos:] = sentinel; V[:, pos:] = sentinel
        Kb, Vb = K.view(np.uint32).copy(), V.view(np.uint32).copy()
        _, dbg = O.attn_block(cfg, g1, wqkv, wo, K, V, pos, x, want_debug=True)
        for arr, before in ((K, Kb), (V, Vb)):
            changed = (arr.view(np.uint32) != before).any(axis=2)
            expect = np.zeros_like(changed); expect[:, pos] = True
            assert np.array_equal(changed, expect)
        assert np.isfinite(dbg["o"]).all()
    cfg, g1, wqkv, wo, K, V, x = _rand_attn(rng)
    with pytest.raises(ValueError):
        O.attn_block(cfg, g1, wqkv, wo, K, V, cfg.max_seq, x)
    with pytest.raises(ValueError):
        O.attn_block(cfg, g1, wqkv, wo, K, V, -1, x)


def test_prefill_equals_successive_decode_steps():
    rng = np.random.default_rng(10)
    cfg, g1, wqkv, wo, K, V, _ = _rand_attn(rng, T=0, max_seq=8)
    n = 5
    X = rng.standard_normal((n, cfg.hidden)).astype(np.float32)
    Kp, Vp = K.copy(), V.copy()
    part_pre = O.attn_block(cfg, g1, wqkv, wo, Kp, Vp, 0, X)
    Kd, Vd = K.copy(), V.copy()
    for i in range(n):
        p = O.attn_block(cfg, g1, wqkv, wo, Kd, Vd, i, X[i])
        np.testing.assert_allclose(part_pre[i], p, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(Kp, Kd); np.testing.assert_array_equal(Vp, Vd)
    # and with a non-empty cache / pos0 > 0
    Kp2, Vp2 = Kd.copy(), Vd.copy(); Kp2[:, 3:] = 0; Vp2[:, 3:] = 0
    part2 = O.attn_block(cfg, g1, wqkv, wo, Kp2, Vp2, 3, X[3:5])
    np.testing.assert_allclose(part2, part_pre[3:5], rtol=1e-13, atol=1e-15)


# ----------------------------------------------------------------------------
# FFN
# ----------------------------------------------------------------------------

def test_swiglu_special_cases():
    rng = np.random.default_rng(11)
    h, s = 32, 24
    cfg = O.ShardCfg(h, 1, 1, 2, s, 4)
    g2 = np.ones(h, np.float32)
    wg = rng.standard_normal((s, h)).astype(np.float32); wu = rng.standard_normal((s, h)).astype(np.float32)
    wd = rng.standard_normal((h, s)).astype(np.float32)
    x = rng.standard_normal(h).astype(np.float32)
    # silu(0) = 0
    assert np.all(O.ffn_block(cfg, g2, np.zeros_like(wg), wu, wd, x) == 0)
    assert np.all(O.ffn_block(cfg, g2, wg, np.zeros_like(wu), wd, x) == 0)
    # silu(t) -> t for large t, -> 0 for very negative t: a gate row that gives +/-50
    xn = O.rmsnorm(x, g2, 1e-5)
    row = (50.0 * xn / (xn @ xn)).astype(np.float32)
    wg2 = np.zeros_like(wg); wg2[0] = row; wg2[1] = -row
    _, dbg = O.ffn_block(cfg, g2, wg2, wu, wd, x, want_debug=True)
    up = wu.astype(np.float64) @ xn
    gt = wg2.astype(np.float64) @ xn
    np.testing.assert_allclose(dbg["act"][0], gt[0] * up[0], rtol=1e-15 + math.exp(-49))
    assert abs(dbg["act"][1]) < 50 * abs(up[1]) * math.exp(-49)
    # silu(1) = 1/(1+e^-1)
    wg3 = np.zeros_like(wg); wg3[2] = (xn / (xn @ xn)).astype(np.float32)
    _, dbg = O.ffn_block(cfg, g2, wg3, wu, wd, x, want_debug=True)
    g = float(wg3[2].astype(np.float64) @ xn)
    np.testing.assert_allclose(dbg["act"][2], g / (1 + math.exp(-g)) * up[2], rtol=1e-14)
    # the down projection is linear in the activation
    p1 = O.ffn_block(cfg, g2, wg, wu, wd, x); p2 = O.ffn_block(cfg, g2, wg, wu, 2 * wd, x)
    np.testing.assert_allclose(p2, 2 * p1, rtol=1e-14)


# ----------------------------------------------------------------------------
# Star reduce
# ----------------------------------------------------------------------------

def test_reduce_order_is_rank_order_then_residual():
    big, one = np.float32(1e8), np.float32(1.0)
    # ((1e8 + 1) + -1e8) = 0 in fp32; any other association gives 1
    assert O.reduce_seq_f32([[big], [one], [-big]])[0] == 0.0
    assert O.reduce_seq_f32([[big], [-big], [one]])[0] == 1.0
    assert O.reduce_seq_f32([[one], [big], [-big]])[0] == 0.0
    # residual is added last: (1e8 + -1e8) + 1 = 1, while 1 joining first would vanish
    assert O.reduce_seq_f32([[big], [-big]], [one])[0] == 1.0
    assert O.reduce_seq_f32([[one], [big]], [-big])[0] == 0.0
    # N = 1
    rng = np.random.default_rng(12)
    p = rng.standard_normal(37).astype(np.float32); r = rng.standard_normal(37).astype(np.float32)
    np.testing.assert_array_equal(O.reduce_seq_f32([p]), p)
    np.testing.assert_array_equal(O.reduce_seq_f32([p], r), p + r)
    # against an fp64 sum: within N ulp-ish, and exact when all addends are small integers
    ps = [rng.integers(-1000, 1000, 64).astype(np.float32) for _ in range(8)]
    np.testing.assert_array_equal(O.reduce_seq_f32(ps, ps[0]), O.reduce_f64(ps, ps[0]).astype(np.float32))
    ps = [rng.standard_normal(64).astype(np.float32) for _ in range(8)]
    np.testing.assert_allclose(O.reduce_seq_f32(ps), O.reduce_f64(ps), rtol=0, atol=8 * 2 ** -23 * 8)


# ----------------------------------------------------------------------------
# Multi-layer driver (Alg. 1 loop body) on the tiny configuration
# ----------------------------------------------------------------------------

def test_tiny_config_layer_stack_matches_unsharded_stack():
    from paper_2410_00531_amd import configs, synth
    m = configs.TINY
    weights, caches, h0 = synth.stack_from_shape(m, seed=0, n_cached=16, max_seq=24)
    cfg = O.ShardCfg(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, 24)
    x = h0
    xd = h0.copy()
    for l in range(m.n_layers):
        sh = weights[l]
        full = {"attn_norm": sh[0]["attn_norm"], "ffn_norm": sh[0]["ffn_norm"]}
        dq, dkv = m.nq_local * m.head_dim, m.nkv_local * m.head_dim
        full["w_q"] = np.concatenate([s["w_qkv"][:dq] for s in sh], 0)
        full["w_k"] = np.concatenate([s["w_qkv"][dq:dq + dkv] for s in sh], 0)
        full["w_v"] = np.concatenate([s["w_qkv"][dq + dkv:] for s in sh], 0)
        full["w_o"] = np.concatenate([s["w_o"] for s in sh], 1)
        full["w_gate"] = np.concatenate([s["w_gate"] for s in sh], 0)
        full["w_up"] = np.concatenate([s["w_up"] for s in sh], 0)
        full["w_down"] = np.concatenate([s["w_down"] for s in sh], 1)
        # the synthetic stack draws separate gains per shard; the identity needs one gain
        for s in sh:
            s["attn_norm"] = full["attn_norm"]; s["ffn_norm"] = full["ffn_norm"]
        Kt = torch.tensor(np.concatenate([c[0] for c in caches[l]], 0))
        Vt = torch.tensor(np.concatenate([c[1] for c in caches[l]], 0))
        _, ref = dense_layer_torch(xd, full, Kt, Vt, 16, m.n_heads, m.n_kv_heads, m.head_dim)
        x, _, _, _ = O.layer_decode(cfg, sh, caches[l], 16, x)
        # fp32 interface roundings on the oracle side: a few ulp of the running magnitude
        np.testing.assert_allclose(x, ref, rtol=0, atol=2e-6 * np.abs(ref).max())
        xd = ref.astype(np.float32)


def test_token_ends_embedding_head_and_token_choice():
    """Ends of the token loop (Sec. 3.1 Step 4; Alg. 1 Preprocess / Postprocess) against library routines,
    closed forms and brute force."""
    rng = np.random.default_rng(31)
    v, h = 53, 40
    w_emb = rng.standard_normal((v, h)).astype(np.float32)
    assert np.array_equal(O.embed_token(w_emb, 17), w_emb[17])
    with pytest.raises(ValueError):
        O.embed_token(w_emb, v)
    g = (1 + 0.1 * rng.standard_normal(h)).astype(np.float32)
    w_head = rng.standard_normal((v, h)).astype(np.float32)
    x = rng.standard_normal(h).astype(np.float32)
    t = lambda a: torch.as_tensor(np.asarray(a), dtype=torch.float64)
    ref = F.linear(t(x) * torch.rsqrt(t(x).pow(2).mean() + 1e-5) * t(g), t(w_head)).numpy()
    logits = O.lm_head(g, w_head, x)
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-12 * np.abs(ref).max())
    # softmax: library routine, sum to one, shift invariance
    p = O.softmax(logits)
    np.testing.assert_allclose(p, torch.softmax(t(logits), 0).numpy(), rtol=1e-13, atol=0)
    assert abs(p.sum() - 1.0) < 1e-14
    np.testing.assert_allclose(O.softmax(logits + 1000.0), p, rtol=1e-10)
    # greedy: numpy's argmax (first occurrence), ties resolved to the lowest index
    assert O.greedy_token(logits) == int(np.argmax(logits))
    assert O.greedy_token(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    # inverse CDF: brute force against the cumulative sums, edges, and the frequencies of many draws
    cdf = np.cumsum(p)
    for u in (0.0, 0.25, 0.5, 0.999999, float(cdf[10]), float(np.nextafter(cdf[10], 0.0))):
        k = O.sample_token(logits, u)
        assert (cdf[k] > u or k == v - 1) and (k == 0 or cdf[k - 1] <= u)
    assert O.sample_token(np.array([0.0, 0.0]), 0.49) == 0 and O.sample_token(np.array([0.0, 0.0]), 0.51) == 1
    us = (np.arange(20000) + 0.5) / 20000
    counts = np.bincount([O.sample_token(logits, float(u)) for u in us], minlength=v)
    np.testing.assert_allclose(counts / 20000, p, atol=1.5 / 20000 + 1e-12)

