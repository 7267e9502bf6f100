"""Whole-token persistent kernel against the per-phase calls on the same inputs
(same arithmetic, different summation order inside the GEMVs: agreement to
1e-5 of the output's max-abs) and against the oracle (1e-4)."""
import numpy as np
import pytest
import torch

from oracle import tpi_oracle as O
from paper_2410_00531_amd import binding as B
from paper_2410_00531_amd import configs, synth
from tpi_testlib import FP32_TOL, GpuShard, ocfg, rel_err

pytestmark = [
    pytest.mark.gpu,
    pytest.mark.skip(reason="this build has no whole-token kernel (tpi_decoder_create returns TPI_EUNSUPPORTED): one run of "
                            "its 8B-shaped case stopped at a grid barrier until the bounded wait gave up, the cause was "
                            "never shown, and the kernel -- slower than the per-stage path anyway -- was taken out"),
]


def _setup(m, n_layers, pos, max_seq, seed, n_ranks, rank):
    weights, caches, h0 = synth.stack_from_shape(m, seed=seed, n_cached=pos, max_seq=max_seq, n_layers=n_layers)
    cfg = B.make_cfg(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, max_seq, m.rms_eps, m.rope_base)
    rng = np.random.default_rng(seed + 99)
    # the other ranks' partials: fixed receive buffers, the same for every layer
    peers_a = [rng.standard_normal(m.hidden).astype(np.float32) * 0.3 for _ in range(n_ranks)]
    peers_f = [rng.standard_normal(m.hidden).astype(np.float32) * 0.3 for _ in range(n_ranks)]
    return weights, caches, h0, cfg, peers_a, peers_f


def _per_phase_gpu(cfg, shards, pos, h0_t, peers_a_t, peers_f_t, rank):
    x = h0_t.clone(); h_attn = torch.empty_like(x); out = torch.empty_like(x)
    for sh in shards:
        B.tpi_shard_layer_decode(cfg, sh.weights, sh.kv, pos, B.TPI_PHASE_ATTN, x, sh.partial, sh.ws)
        pa = [sh.partial if i == rank else p for i, p in enumerate(peers_a_t)]
        B.tpi_star_reduce(pa, x, h_attn)
        B.tpi_shard_layer_decode(cfg, sh.weights, None, pos, B.TPI_PHASE_FFN, h_attn, sh.partial, sh.ws)
        pf = [sh.partial if i == rank else p for i, p in enumerate(peers_f_t)]
        B.tpi_star_reduce(pf, h_attn, out)
        x = out.clone()
    torch.cuda.synchronize()
    return x


def _oracle(cfg, weights, caches, pos, h0, peers_a, peers_f, rank):
    oc = ocfg(cfg)
    x = h0
    for l, w in enumerate(weights):
        s = w[0]; K, V = caches[l][0]
        pa = O.attn_block(oc, s["attn_norm"], s["w_qkv"], s["w_o"], K, V, pos, x).astype(np.float32)
        h_attn = O.reduce_seq_f32([pa if i == rank else p for i, p in enumerate(peers_a)], x)
        pf = O.ffn_block(oc, s["ffn_norm"], s["w_gate"], s["w_up"], s["w_down"], h_attn).astype(np.float32)
        x = O.reduce_seq_f32([pf if i == rank else p for i, p in enumerate(peers_f)], h_attn)
    return x


@pytest.mark.parametrize("name,n_layers,pos,n_ranks,rank,tokens", [
    ("tiny", 2, 16, 2, 0, 1),
    ("tiny", 2, 16, 2, 1, 3),
    ("tiny", 5, 0, 1, 0, 2),
    ("llama3.1-8b-shaped-tp4", 3, 512, 4, 2, 2),
    ("llama2-70b-shaped-tp8", 3, 1024, 8, 0, 2),
])
def test_decoder_matches_per_phase_calls_and_oracle(name, n_layers, pos, n_ranks, rank, tokens):
    m = configs.BY_NAME[name]
    max_seq = pos + tokens + 4
    weights, caches, h0, cfg, peers_a, peers_f = _setup(m, n_layers, pos, max_seq, 7, n_ranks, rank)
    pa_t = [torch.from_numpy(p).cuda() for p in peers_a]
    pf_t = [torch.from_numpy(p).cuda() for p in peers_f]
    h0_t = torch.from_numpy(h0).cuda()
    ref_sh = [GpuShard(cfg, weights[l][0], *caches[l][0]) for l in range(n_layers)]
    dec_sh = [GpuShard(cfg, weights[l][0], *caches[l][0]) for l in range(n_layers)]
    dec = B.Decoder(cfg, [s.weights for s in dec_sh], [s.kv for s in dec_sh], rank,
                    pa_t if n_ranks > 1 else None, pf_t if n_ranks > 1 else None)
    assert dec.grid >= 1
    out = torch.empty_like(h0_t)
    o_caches = [[(caches[l][0][0].copy(), caches[l][0][1].copy())] for l in range(n_layers)]
    for t in range(tokens):
        ref = _per_phase_gpu(cfg, ref_sh, pos + t, h0_t, pa_t, pf_t, rank)
        dec.token(pos + t, h0_t, out)
        dec.status()
        e = rel_err(out.cpu().numpy(), ref.cpu().numpy())
        assert e <= 1e-5, f"token {t}: persistent kernel differs from the per-phase calls by {e:.2e}"
        for a, b in zip(dec_sh, ref_sh):
            # same slots written, values equal up to the summation order
            assert torch.equal(a.K != 0, b.K != 0) and torch.equal(a.V != 0, b.V != 0)
            assert rel_err(a.K.cpu().numpy(), b.K.cpu().numpy()) <= 1e-5
            assert rel_err(a.V.cpu().numpy(), b.V.cpu().numpy()) <= 1e-5
        want = _oracle(cfg, weights, o_caches, pos + t, h0, peers_a, peers_f, rank)
        assert rel_err(out.cpu().numpy(), want) <= FP32_TOL
    dec.destroy()


def test_decoder_rejects_bad_arguments():
    m = configs.TINY
    cfg = B.make_cfg(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, 8)
    w, K, V = synth.make_layer_shard(np.random.default_rng(0), m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local), \
        np.zeros((m.nkv_local, 8, m.head_dim), np.float32), np.zeros((m.nkv_local, 8, m.head_dim), np.float32)
    sh = GpuShard(cfg, w, K, V)
    dec = B.Decoder(cfg, [sh.weights], [sh.kv])
    x = torch.zeros(m.hidden, device="cuda"); y = torch.empty_like(x)
    for bad_pos in (-1, 8):
        with pytest.raises(B.TpiError) as ei:
            dec.token(bad_pos, x, y)
        assert ei.value.code == B.TPI_EINVAL
    with pytest.raises(B.TpiError) as ei:
        dec.token(0, None, y)
    assert ei.value.code == B.TPI_EINVAL
    dec.token(0, x, y); dec.status()
    dec.destroy()
    # a shape the whole-token kernel is not compiled for is reported, not guessed
    odd = B.make_cfg(2056, 1, 1, 24, 2056, 8)
    with pytest.raises(B.TpiError) as ei:
        B.Decoder(odd, [sh.weights], [sh.kv])
    assert ei.value.code == B.TPI_EUNSUPPORTED
