"""GPU parity of the fp32 decode path against the CPU oracle, through the C ABI.
Tolerance: max |gpu - oracle| <= 1e-4 * max |oracle| (fp32 paths); cache slot
indexing and the star reduce are bit-exact."""
import numpy as np
import pytest
import torch

from oracle import tpi_oracle as O
from paper_2410_00531_amd import binding as B
from paper_2410_00531_amd import configs, synth
from tpi_testlib import (FP32_TOL, GpuShard, check_attn_phase, check_ffn_phase, gpu_layer_decode,
                         ocfg, random_shard_np, rel_err)

pytestmark = pytest.mark.gpu


def _cfg_of(m: configs.ModelShape, max_seq):
    return B.make_cfg(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, max_seq,
                      m.rms_eps, m.rope_base)


def test_tiny_config_two_layers_two_shards():
    """The tiny 2-layer, 2-shard workload: teacher-forced per-shard parity and the free-running stack."""
    m = configs.TINY
    pos, max_seq = 16, 24
    weights, caches, h0 = synth.stack_from_shape(m, seed=0, n_cached=pos, max_seq=max_seq)
    cfg = _cfg_of(m, max_seq)
    oc = ocfg(cfg)
    # oracle, free running
    xo = h0.copy()
    o_states = []
    o_caches = [[(K.copy(), V.copy()) for K, V in row] for row in caches]
    for l in range(m.n_layers):
        h_ffn, h_attn, pa, pf = O.layer_decode(oc, weights[l], o_caches[l], pos, xo)
        o_states.append((xo.copy(), h_attn, h_ffn, pa, pf))
        xo = h_ffn
    # GPU, free running
    x = torch.from_numpy(h0).cuda()
    h_attn_t = torch.empty_like(x); h_out_t = torch.empty_like(x)
    for l in range(m.n_layers):
        shards = [GpuShard(cfg, weights[l][r], *caches[l][r]) for r in range(m.n_shards)]
        gpu_layer_decode(cfg, shards, pos, x, h_attn_t, h_out_t, batched=(l % 2 == 0))
        torch.cuda.synchronize()
        x_in, h_attn, h_ffn, pa, pf = o_states[l]
        assert rel_err(h_attn_t.cpu().numpy(), h_attn) <= FP32_TOL
        assert rel_err(h_out_t.cpu().numpy(), h_ffn) <= FP32_TOL
        for r in range(m.n_shards):
            assert rel_err(shards[r].partial.cpu().numpy(), pf[r]) <= FP32_TOL
            Kg = shards[r].K.cpu().numpy(); Ko = o_caches[l][r][0]
            assert rel_err(Kg[:, pos], Ko[:, pos]) <= FP32_TOL
            assert np.array_equal(Kg[:, :pos], Ko[:, :pos])
        x = h_out_t.clone()
    # teacher-forced, per shard and phase, with sentinel-checked cache writes
    for l in range(m.n_layers):
        x_in, h_attn, _, _, _ = o_states[l]
        for r in range(m.n_shards):
            check_attn_phase(cfg, weights[l][r], *caches[l][r], pos, x_in)
            check_ffn_phase(cfg, weights[l][r], h_attn)


@pytest.mark.parametrize("h,nq,nkv,d,sl", [
    (256, 2, 2, 64, 344),      # tiny shard
    (264, 3, 1, 32, 100),      # group of 3 (padded head tile), short rows, ragged tails
    (1032, 4, 2, 128, 1000),   # rows longer than one 1024-float pass, ragged
    (512, 16, 1, 64, 520),     # group of 16: two head tiles of 8
    (384, 2, 1, 256, 256),     # widest head
    (128, 5, 5, 8, 64),        # narrowest head, MHA, odd head count
    (2056, 1, 1, 24, 2056),    # head_dim not a power of two (padded lanes)
])
def test_ragged_shapes(h, nq, nkv, d, sl):
    rng = np.random.default_rng(h + nq + d)
    pos, max_seq = 37, 40
    cfg = B.make_cfg(h, nq, nkv, d, sl, max_seq)
    w, K, V = random_shard_np(rng, cfg, pos)
    x = rng.standard_normal(h).astype(np.float32)
    check_attn_phase(cfg, w, K, V, pos, x)
    check_ffn_phase(cfg, w, x)


def _random_decode_shapes(n, seed):
    """Seeded random shard shapes inside the documented limits: hidden and FFN width multiples of 4, head
    sizes even multiples of 4 up to 256, any group size, positions anywhere in the cache."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        d = int(rng.choice([4, 8, 12, 16, 24, 32, 40, 64, 80, 96, 128, 160, 192, 256]))
        nkv = int(rng.integers(1, 4))
        G = int(rng.choice([1, 1, 2, 3, 4, 5, 8, 9, 16]))
        if G * nkv * d > 2048:
            G = max(1, 2048 // (nkv * d))
        h = 4 * int(rng.integers(1, 600))
        sl = 4 * int(rng.integers(1, 700))
        max_seq = int(rng.integers(1, 700))
        pos = int(rng.integers(0, max_seq))
        out.append((h, G * nkv, nkv, d, sl, pos, max_seq))
    return out


@pytest.mark.parametrize("h,nq,nkv,d,sl,pos,max_seq", _random_decode_shapes(24, 2024))
def test_random_shapes_both_phases(h, nq, nkv, d, sl, pos, max_seq):
    rng = np.random.default_rng(h * 7 + sl + pos)
    cfg = B.make_cfg(h, nq, nkv, d, sl, max_seq)
    w, K, V = random_shard_np(rng, cfg, pos)
    x = rng.standard_normal(h).astype(np.float32)
    check_attn_phase(cfg, w, K, V, pos, x)
    check_ffn_phase(cfg, w, x)


@pytest.mark.parametrize("h,nq,nkv,d,sl", [
    (16384, 2, 1, 64, 128),      # the longest row the QKV and gate/up stages are built for (16 passes of 1024)
    (256, 128, 1, 128, 16384),   # the same for the output projection (n_q * d = 16384) and the down projection
])
def test_longest_rows(h, nq, nkv, d, sl):
    rng = np.random.default_rng(h + sl)
    pos, max_seq = 5, 8
    cfg = B.make_cfg(h, nq, nkv, d, sl, max_seq)
    w, K, V = random_shard_np(rng, cfg, pos)
    x = rng.standard_normal(h).astype(np.float32)
    check_attn_phase(cfg, w, K, V, pos, x)
    check_ffn_phase(cfg, w, x)


@pytest.mark.parametrize("pos,max_seq", [
    (0, 1), (0, 8), (1, 8), (63, 64), (64, 65), (65, 130), (127, 128), (2047, 2048), (2048, 2100),
    (2111, 2112), (4500, 4501),
])
def test_positions_tiles_splits_and_last_slot(pos, max_seq):
    """Empty cache, tile edges (64), split edges (32 splits), multi-tile chunks
    with the running softmax (pos > 2048), and the last slot of the cache."""
    rng = np.random.default_rng(pos)
    cfg = B.make_cfg(256, 8, 2, 64, 64, max_seq)
    # larger keys make the softmax peaky, so the running maximum matters
    w, K, V = random_shard_np(rng, cfg, pos, kv_scale=3.0)
    w["w_qkv"] *= 8
    x = rng.standard_normal(256).astype(np.float32)
    check_attn_phase(cfg, w, K, V, pos, x)


def test_rope_position_zero_is_identity_on_gpu():
    """At pos 0 the stored key equals the unrotated projection bit for bit: the
    same call with rope_base changed must write identical bits."""
    rng = np.random.default_rng(3)
    outs = []
    for base in (10000.0, 500000.0):
        cfg = B.make_cfg(256, 2, 2, 64, 64, 4, rope_base=base)
        w, K, V = random_shard_np(np.random.default_rng(3), cfg, 0)
        sh = GpuShard(cfg, w, K, V)
        x = torch.from_numpy(np.random.default_rng(4).standard_normal(256).astype(np.float32)).cuda()
        B.tpi_shard_layer_decode(cfg, sh.weights, sh.kv, 0, B.TPI_PHASE_ATTN, x, sh.partial, sh.ws)
        torch.cuda.synchronize()
        outs.append((sh.K.cpu().numpy().copy(), sh.partial.cpu().numpy().copy()))
    assert np.array_equal(outs[0][0].view(np.uint32), outs[1][0].view(np.uint32))
    assert np.array_equal(outs[0][1].view(np.uint32), outs[1][1].view(np.uint32))


def test_large_positions_keep_rope_phase():
    """Angles of thousands of radians: the rotation must still match fp64."""
    rng = np.random.default_rng(5)
    pos, max_seq = 100_000, 100_001
    cfg = B.make_cfg(128, 1, 1, 64, 64, max_seq)
    w, K, V = random_shard_np(rng, cfg, 0)
    K[:, :pos] = rng.standard_normal((1, pos, 64), dtype=np.float32)
    V[:, :pos] = rng.standard_normal((1, pos, 64), dtype=np.float32)
    x = rng.standard_normal(128).astype(np.float32)
    check_attn_phase(cfg, w, K, V, pos, x, sentinel=False)


@pytest.mark.parametrize("n", [5, B.TPI_MAX_BATCH_SHARDS])
def test_batched_call_equals_single_calls_bitwise(n):
    rng = np.random.default_rng(6)
    cfg = B.make_cfg(512, 4, 2, 64, 256, 80)
    pos = 70
    data = [random_shard_np(rng, cfg, pos) for _ in range(n)]
    x = torch.from_numpy(rng.standard_normal(512).astype(np.float32)).cuda()
    a = [GpuShard(cfg, *d) for d in data]
    b = [GpuShard(cfg, *d) for d in data]
    for phase in (B.TPI_PHASE_ATTN, B.TPI_PHASE_FFN):
        B.tpi_shards_layer_decode(cfg, [s.weights for s in a], [s.kv for s in a], pos, phase, x,
                                  [s.partial for s in a], [s.ws for s in a])
        for s in b:
            B.tpi_shard_layer_decode(cfg, s.weights, s.kv, pos, phase, x, s.partial, s.ws)
        torch.cuda.synchronize()
        for sa, sb in zip(a, b):
            assert torch.equal(sa.partial, sb.partial)
            assert torch.equal(sa.K, sb.K) and torch.equal(sa.V, sb.V)


def test_reduce_folded_into_the_phase_is_bitwise_the_two_call_sequence():
    rng = np.random.default_rng(21)
    for (h, nq, nkv, d, sl, n, rank) in ((256, 2, 2, 64, 344, 2, 1), (1032, 4, 2, 128, 1000, 5, 0), (512, 8, 1, 64, 520, 1, 0)):
        cfg = B.make_cfg(h, nq, nkv, d, sl, 40)
        pos = 33
        w, K, V = random_shard_np(rng, cfg, pos)
        peers = [torch.from_numpy(rng.standard_normal(h).astype(np.float32)).cuda() for _ in range(n)]
        x = torch.from_numpy(rng.standard_normal(h).astype(np.float32)).cuda()
        a = GpuShard(cfg, w, K, V); b = GpuShard(cfg, w, K, V)
        for phase in (B.TPI_PHASE_ATTN, B.TPI_PHASE_FFN):
            B.tpi_shard_layer_decode(cfg, a.weights, a.kv, pos, phase, x, a.partial, a.ws)
            want = torch.empty(h, device="cuda")
            B.tpi_star_reduce([a.partial if i == rank else p for i, p in enumerate(peers)], x, want)
            got = torch.empty(h, device="cuda")
            B.tpi_shard_layer_decode_reduce(cfg, b.weights, b.kv, pos, phase, x, rank, peers, got, b.ws)
            torch.cuda.synchronize()
            assert torch.equal(got, want)
            # in place on the hidden state
            xin = x.clone()
            B.tpi_shard_layer_decode_reduce(cfg, b.weights, b.kv, pos, phase, xin, rank, peers, xin, b.ws)
            torch.cuda.synchronize()
            assert torch.equal(xin, want)


@pytest.mark.parametrize("h,nq,nkv,d,sl,n", [
    (256, 2, 2, 64, 344, 2),          # tiny
    (1032, 4, 2, 128, 1000, 5),       # ragged rows: the last row group is short, K not a multiple of 1024
    (512, 8, 1, 64, 520, 1),          # one rank: the reduce is only the shortcut
    (8192, 8, 1, 128, 3584, 8),       # the 70B-shaped shard, 8 ranks
    (4096, 8, 2, 128, 3584, 4),       # the 8B-shaped shard, 4 ranks
    (264, 2, 1, 96, 5000, B.TPI_MAX_BATCH_SHARDS),
])
def test_batched_phase_with_reduce_is_bitwise_the_two_call_sequence(h, nq, nkv, d, sl, n):
    """tpi_shards_layer_decode_reduce: all ranks' row-parallel products and their star reduce in the last stage's
    workgroups.  Must equal tpi_shards_layer_decode + tpi_star_reduce bit for bit, and write the same cache slots."""
    rng = np.random.default_rng(h + n)
    cfg = B.make_cfg(h, nq, nkv, d, sl, 40)
    pos = 33
    data = [random_shard_np(rng, cfg, pos) for _ in range(n)]
    x = torch.from_numpy(rng.standard_normal(h).astype(np.float32)).cuda()
    a = [GpuShard(cfg, *dd) for dd in data]
    b = [GpuShard(cfg, *dd) for dd in data]
    for phase in (B.TPI_PHASE_ATTN, B.TPI_PHASE_FFN):
        B.tpi_shards_layer_decode(cfg, [s_.weights for s_ in a], [s_.kv for s_ in a], pos, phase, x,
                                  [s_.partial for s_ in a], [s_.ws for s_ in a])
        want = torch.empty(h, device="cuda")
        B.tpi_star_reduce([s_.partial for s_ in a], x, want)
        got = torch.full((h,), float("nan"), device="cuda")
        B.tpi_shards_layer_decode_reduce(cfg, [s_.weights for s_ in b], [s_.kv for s_ in b], pos, phase, x, got,
                                         [s_.ws for s_ in b])
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        for sa, sb in zip(a, b):
            assert torch.equal(sa.K, sb.K) and torch.equal(sa.V, sb.V)


def test_token_captured_in_a_graph_replays_to_the_eager_result():
    """The decode entry points only enqueue kernels on the caller's stream, so a whole token (phases and
    reduces of several layers, batched and folded variants) can be captured once and replayed.  Every replay,
    with eager work and synchronisations in between, must reproduce the eager token bit for bit."""
    rng = np.random.default_rng(77)
    n_layers, n_sh, h, pos = 3, 2, 512, 21
    cfg = B.make_cfg(h, 4, 2, 64, 264, 40)
    layers = [[GpuShard(cfg, *random_shard_np(rng, cfg, pos)) for _ in range(n_sh)] for _ in range(n_layers)]
    x0 = torch.from_numpy(rng.standard_normal(h).astype(np.float32)).cuda()
    hs = [torch.empty(h, device="cuda") for _ in range(3)]

    def token(folded):
        src, mid, dst = x0, hs[0], hs[1]
        for sh in layers:
            for phase, a, b in ((B.TPI_PHASE_ATTN, src, mid), (B.TPI_PHASE_FFN, mid, dst)):
                if folded:   # shard 1's partial first, then shard 0 with the reduce in its epilogue
                    B.tpi_shard_layer_decode(cfg, sh[1].weights, sh[1].kv, pos, phase, a, sh[1].partial, sh[1].ws)
                    B.tpi_shard_layer_decode_reduce(cfg, sh[0].weights, sh[0].kv, pos, phase, a, 0,
                                                    [sh[0].partial, sh[1].partial], b, sh[0].ws)
                else:
                    B.tpi_shards_layer_decode(cfg, [s.weights for s in sh], [s.kv for s in sh], pos, phase, a,
                                              [s.partial for s in sh], [s.ws for s in sh])
                    B.tpi_star_reduce([s.partial for s in sh], a, b)
            src, dst = dst, (hs[2] if dst is hs[1] else hs[1])
        return src

    for folded in (False, True):
        want = token(folded).clone()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            out = token(folded)
        for rep in range(3):
            for t in hs: t.fill_(float("nan"))           # eager work between the replays
            for sh in layers:
                for s in sh: s.partial.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, want), f"replay {rep}, folded={folded}"


def test_8b_shaped_layer_all_shards():
    """The 8B-shaped 4-way shard: one layer, N = 4, KV length 512."""
    m = configs.LLAMA31_8B_TP4
    pos, max_seq = 512, 520
    weights, caches, h0 = synth.stack_from_shape(m, seed=1, n_cached=pos, max_seq=max_seq, n_layers=1)
    cfg = _cfg_of(m, max_seq)
    shards = [GpuShard(cfg, weights[0][r], *caches[0][r]) for r in range(m.n_shards)]
    x = torch.from_numpy(h0).cuda()
    h_attn_t = torch.empty_like(x); h_out_t = torch.empty_like(x)
    gpu_layer_decode(cfg, shards, pos, x, h_attn_t, h_out_t)
    torch.cuda.synchronize()
    h_ffn, h_attn, pa, pf = O.layer_decode(ocfg(cfg), weights[0], caches[0], pos, h0)
    assert rel_err(h_attn_t.cpu().numpy(), h_attn) <= FP32_TOL
    assert rel_err(h_out_t.cpu().numpy(), h_ffn) <= FP32_TOL
    for r in range(m.n_shards):
        assert rel_err(shards[r].partial.cpu().numpy(), pf[r]) <= FP32_TOL
        assert rel_err(shards[r].K.cpu().numpy()[:, pos], caches[0][r][0][:, pos]) <= FP32_TOL


def test_70b_shaped_layer_all_shards():
    """The 70B-shaped 8-way shard in the launch configuration the benchmark times (8 shards batched, KV
    length 1024): weights drawn on the device, the oracle gets the same bytes."""
    m = configs.LLAMA2_70B_TP8
    pos, max_seq = 1024, 1032
    cfg = _cfg_of(m, max_seq)
    gen = torch.Generator(device="cuda"); gen.manual_seed(70)
    shapes = synth.shard_tensor_shapes(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local)
    shards, host = [], []
    for r in range(m.n_shards):
        w = {}
        for name, shp in shapes.items():
            t = torch.randn(shp, generator=gen, device="cuda", dtype=torch.float32) * synth.WEIGHT_STD
            if name.endswith("_norm"):
                t += 1.0
            w[name] = t
        K = torch.zeros((m.nkv_local, max_seq, m.head_dim), device="cuda")
        V = torch.zeros_like(K)
        K[:, :pos] = torch.randn((m.nkv_local, pos, m.head_dim), generator=gen, device="cuda")
        V[:, :pos] = torch.randn((m.nkv_local, pos, m.head_dim), generator=gen, device="cuda")
        host.append(({k: v.cpu().numpy() for k, v in w.items()}, K.cpu().numpy(), V.cpu().numpy()))
        sh = GpuShard.__new__(GpuShard)
        sh.cfg = cfg; sh.w = w; sh.K = K; sh.V = V
        sh.weights = B.make_weights(w); sh.kv = B.make_kv(K, V)
        sh.partial = torch.empty(m.hidden, device="cuda")
        sh.ws = torch.full((B.tpi_workspace_bytes(cfg, 1) // 4,), float("nan"), device="cuda")
        shards.append(sh)
    x = torch.randn(m.hidden, generator=gen, device="cuda")
    h_attn_t = torch.empty_like(x); h_out_t = torch.empty_like(x)
    gpu_layer_decode(cfg, shards, pos, x, h_attn_t, h_out_t)
    torch.cuda.synchronize()
    oc = ocfg(cfg)
    h0 = x.cpu().numpy()
    wl = [h[0] for h in host]; kv = [(h[1], h[2]) for h in host]
    h_ffn, h_attn, pa, pf = O.layer_decode(oc, wl, kv, pos, h0)
    assert rel_err(h_attn_t.cpu().numpy(), h_attn) <= FP32_TOL
    assert rel_err(h_out_t.cpu().numpy(), h_ffn) <= FP32_TOL
    for r in range(m.n_shards):
        assert rel_err(shards[r].partial.cpu().numpy(), pf[r]) <= FP32_TOL
        Kg = shards[r].K.cpu().numpy()
        assert rel_err(Kg[:, pos], kv[r][0][:, pos]) <= FP32_TOL
        assert np.array_equal(Kg[:, :pos], kv[r][0][:, :pos]) and not Kg[:, pos + 1:].any()
    # The entry point the benchmark's headline step calls, at its full size, directly against the oracle: all 8
    # shards per launch with both star reduces folded into the row-parallel kernels (the caches take the same
    # slot again, so the run above does not change its input).
    ws = [s.weights for s in shards]; kvs = [s.kv for s in shards]; wss = [s.ws for s in shards]
    for s in shards:
        s.ws.fill_(float("nan"))
    h_attn2 = torch.full_like(x, float("nan")); h_out2 = torch.full_like(x, float("nan"))
    B.tpi_shards_layer_decode_reduce(cfg, ws, kvs, pos, B.TPI_PHASE_ATTN, x, h_attn2, wss)
    B.tpi_shards_layer_decode_reduce(cfg, ws, None, pos, B.TPI_PHASE_FFN, h_attn2, h_out2, wss)
    torch.cuda.synchronize()
    e_attn, e_ffn = rel_err(h_attn2.cpu().numpy(), h_attn), rel_err(h_out2.cpu().numpy(), h_ffn)
    print(f"70B-shaped layer, 8 shards, KV 1024, reduces folded in: H_attn rel err {e_attn:.2e}, H_ffn {e_ffn:.2e}", flush=True)
    assert e_attn <= FP32_TOL and e_ffn <= FP32_TOL
    for r in range(m.n_shards):
        Kg, Vg = shards[r].K.cpu().numpy(), shards[r].V.cpu().numpy()
        assert rel_err(Kg[:, pos], kv[r][0][:, pos]) <= FP32_TOL and rel_err(Vg[:, pos], kv[r][1][:, pos]) <= FP32_TOL
        assert np.array_equal(Kg[:, :pos], kv[r][0][:, :pos]) and not Kg[:, pos + 1:].any()


def test_70b_shaped_stack_two_tokens_free_running_and_teacher_forced():
    """Six layers of the 70B-shaped 8-way stack (8 shards batched per launch, KV length 1024), two
    tokens in a row.  Free-running: the device feeds itself and is compared with the oracle feeding
    itself, layer by layer.  Teacher-forced: every device layer is also run from the oracle's input of
    that layer, so a drift of the free-running comparison cannot hide behind accumulated error."""
    m = configs.LLAMA2_70B_TP8
    L, pos0, n_tok, max_seq = 6, 1024, 2, 1032
    cfg = _cfg_of(m, max_seq)
    oc = ocfg(cfg)
    gen = torch.Generator(device="cuda"); gen.manual_seed(7070)
    shapes = synth.shard_tensor_shapes(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local)
    layers, host = [], []
    for l in range(L):
        shards, hs = [], []
        for r in range(m.n_shards):
            w = {}
            for name, shp in shapes.items():
                t = torch.randn(shp, generator=gen, device="cuda", dtype=torch.float32) * synth.WEIGHT_STD
                if name.endswith("_norm"):
                    t += 1.0
                w[name] = t
            K = torch.zeros((m.nkv_local, max_seq, m.head_dim), device="cuda")
            V = torch.zeros_like(K)
            K[:, :pos0] = torch.randn((m.nkv_local, pos0, m.head_dim), generator=gen, device="cuda")
            V[:, :pos0] = torch.randn((m.nkv_local, pos0, m.head_dim), generator=gen, device="cuda")
            hs.append(({k: v.cpu().numpy() for k, v in w.items()}, K.cpu().numpy(), V.cpu().numpy()))
            sh = GpuShard.__new__(GpuShard)
            sh.cfg = cfg; sh.w = w; sh.K = K; sh.V = V
            sh.weights = B.make_weights(w); sh.kv = B.make_kv(K, V)
            sh.partial = torch.empty(m.hidden, device="cuda")
            sh.ws = torch.full((B.tpi_workspace_bytes(cfg, 1) // 4,), float("nan"), device="cuda")
            shards.append(sh)
        layers.append(shards); host.append(hs)
    # a second set of device caches for the teacher-forced runs (they must not disturb the free-running ones)
    tf_kv = [[(s.K.clone(), s.V.clone()) for s in shards] for shards in layers]
    h_attn_t = torch.empty(m.hidden, device="cuda"); out_t = torch.empty(m.hidden, device="cuda")
    tf_attn = torch.empty_like(h_attn_t); tf_out = torch.empty_like(out_t)
    x0 = torch.randn(m.hidden, generator=gen, device="cuda")
    worst_free = worst_tf = 0.0
    for t in range(n_tok):
        pos = pos0 + t
        x_gpu = x0 + float(t)                       # a different input per token
        x_orc = x_gpu.cpu().numpy()
        for l in range(L):
            shards = layers[l]
            gpu_layer_decode(cfg, shards, pos, x_gpu, h_attn_t, out_t)
            # teacher-forced: same layer, the oracle's input, separate caches
            saved = [(s.K, s.V, s.kv) for s in shards]
            for s, (Kc, Vc) in zip(shards, tf_kv[l]):
                s.K, s.V, s.kv = Kc, Vc, B.make_kv(Kc, Vc)
            gpu_layer_decode(cfg, shards, pos, torch.from_numpy(x_orc).cuda(), tf_attn, tf_out)
            for s, (Kc, Vc, kvs) in zip(shards, saved):
                s.K, s.V, s.kv = Kc, Vc, kvs
            torch.cuda.synchronize()
            wl = [h[0] for h in host[l]]; kv = [(h[1], h[2]) for h in host[l]]
            h_ffn, h_attn, pa, pf = O.layer_decode(oc, wl, kv, pos, x_orc)
            worst_tf = max(worst_tf, rel_err(tf_attn.cpu().numpy(), h_attn), rel_err(tf_out.cpu().numpy(), h_ffn))
            worst_free = max(worst_free, rel_err(h_attn_t.cpu().numpy(), h_attn), rel_err(out_t.cpu().numpy(), h_ffn))
            for r in range(m.n_shards):
                assert rel_err(shards[r].K.cpu().numpy()[:, pos], kv[r][0][:, pos]) <= FP32_TOL
            x_gpu = out_t.clone()
            x_orc = h_ffn
    print(f"70B-shaped stack, {L} layers x {n_tok} tokens: worst rel err teacher-forced {worst_tf:.2e}, "
          f"free-running {worst_free:.2e}", flush=True)
    assert worst_tf <= FP32_TOL
    assert worst_free <= FP32_TOL


# ----------------------------------------------------------------------------
# Star reduce: bit-exact
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("n,length", [(1, 5), (2, 256), (8, 8192), (8, 8191), (3, 3), (64, 1000),
                                      (8, 512 * 8192)])
def test_star_reduce_bit_exact(n, length):
    rng = np.random.default_rng(n * 1000 + length)
    ps = [(rng.standard_normal(length) * 10 ** rng.uniform(-3, 3, length)).astype(np.float32) for _ in range(n)]
    res = rng.standard_normal(length).astype(np.float32)
    tp = [torch.from_numpy(p).cuda() for p in ps]
    tr = torch.from_numpy(res).cuda()
    out = torch.empty(length, device="cuda")
    B.tpi_star_reduce(tp, tr, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint32), O.reduce_seq_f32(ps, res).view(np.uint32))
    B.tpi_star_reduce(tp, None, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint32), O.reduce_seq_f32(ps).view(np.uint32))


def test_star_reduce_order_unaligned_and_aliasing():
    big, one = 1e8, 1.0
    mk = lambda v: torch.full((8,), v, device="cuda", dtype=torch.float32)
    out = torch.empty(8, device="cuda")
    B.tpi_star_reduce([mk(big), mk(one), mk(-big)], None, out); torch.cuda.synchronize()
    assert (out == 0).all()
    B.tpi_star_reduce([mk(big), mk(-big), mk(one)], None, out); torch.cuda.synchronize()
    assert (out == 1).all()
    B.tpi_star_reduce([mk(big), mk(-big)], mk(one), out); torch.cuda.synchronize()
    assert (out == 1).all()
    B.tpi_star_reduce([mk(one), mk(big)], mk(-big), out); torch.cuda.synchronize()
    assert (out == 0).all()
    # pointers off the 16-byte grid take the scalar path, same bits
    rng = np.random.default_rng(0)
    ps = [rng.standard_normal(1001).astype(np.float32) for _ in range(4)]
    buf = [torch.from_numpy(np.concatenate([[0], p]).astype(np.float32)).cuda() for p in ps]
    outb = torch.empty(1002, device="cuda")
    B.tpi_star_reduce([b[1:] for b in buf], None, outb[1:], length=1001); torch.cuda.synchronize()
    assert np.array_equal(outb[1:].cpu().numpy().view(np.uint32), O.reduce_seq_f32(ps).view(np.uint32))
    # out may alias the residual (H is updated in place)
    tp = [torch.from_numpy(p).cuda() for p in ps]
    res = torch.from_numpy(ps[0].copy()).cuda()
    B.tpi_star_reduce(tp, res, res); torch.cuda.synchronize()
    assert np.array_equal(res.cpu().numpy().view(np.uint32), O.reduce_seq_f32(ps, ps[0]).view(np.uint32))
    # zero length is a no-op
    B.tpi_star_reduce(tp, None, out, length=0)


def test_layer_with_uneven_shares_matches_oracle():
    """Sec. 3.1 lets device i hold a proportion p_i of the heads and FFN columns.  Three shards with
    4 / 2 / 2 query heads, 2 / 1 / 1 KV heads and 1100 / 600 / 348 FFN columns, each with its own shard
    configuration, run phase by phase through the library; partials, reduces and caches must match the
    oracle run on the same shards."""
    h, d, max_seq, pos = 512, 64, 40, 33
    split = [(4, 2, 1100), (2, 1, 600), (2, 1, 348)]
    rng = np.random.default_rng(808)
    x = rng.standard_normal(h).astype(np.float32)
    cfgs, ws, caches, gsh = [], [], [], []
    for nq, nkv, sl in split:
        cfg = B.make_cfg(h, nq, nkv, d, sl, max_seq)
        w, K, V = random_shard_np(rng, cfg, pos)
        cfgs.append(cfg); ws.append(w); caches.append((K.copy(), V.copy()))
        gsh.append(GpuShard(cfg, w, K, V))
    xt = torch.from_numpy(x).cuda()
    h_attn = torch.empty_like(xt); h_out = torch.empty_like(xt)
    for cfg, s in zip(cfgs, gsh):
        B.tpi_shard_layer_decode(cfg, s.weights, s.kv, pos, B.TPI_PHASE_ATTN, xt, s.partial, s.ws)
    B.tpi_star_reduce([s.partial for s in gsh], xt, h_attn)
    for cfg, s in zip(cfgs, gsh):
        B.tpi_shard_layer_decode(cfg, s.weights, None, pos, B.TPI_PHASE_FFN, h_attn, s.partial, s.ws)
    B.tpi_star_reduce([s.partial for s in gsh], h_attn, h_out)
    torch.cuda.synchronize()
    pa = [O.attn_block(ocfg(c), w["attn_norm"], w["w_qkv"], w["w_o"], kv[0], kv[1], pos, x).astype(np.float32)
          for c, w, kv in zip(cfgs, ws, caches)]
    ref_attn = O.reduce_seq_f32(pa, x)
    pf = [O.ffn_block(ocfg(c), w["ffn_norm"], w["w_gate"], w["w_up"], w["w_down"], ref_attn).astype(np.float32)
          for c, w in zip(cfgs, ws)]
    ref_out = O.reduce_seq_f32(pf, ref_attn)
    assert rel_err(h_attn.cpu().numpy(), ref_attn) <= FP32_TOL
    assert rel_err(h_out.cpu().numpy(), ref_out) <= FP32_TOL
    for s, (Ko, Vo) in zip(gsh, caches):
        assert rel_err(s.K.cpu().numpy()[:, pos], Ko[:, pos]) <= FP32_TOL
        assert rel_err(s.V.cpu().numpy()[:, pos], Vo[:, pos]) <= FP32_TOL

