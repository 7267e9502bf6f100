"""GPU parity of the bf16 prefill path (matrix cores) against the CPU oracle.
Inputs and weights are bf16 values (the oracle gets exactly those, widened);
tolerance 2e-2 of the oracle output's max-abs; cache slot set is exact."""
import numpy as np
import pytest
import torch

from oracle import tpi_oracle as O
from paper_2410_00531_amd import binding as B
from paper_2410_00531_amd import configs, synth
from tpi_testlib import BF16_TOL, rel_err

pytestmark = pytest.mark.gpu


def _bf16_t(x_np):
    """float32 numpy array that already lies on the bf16 grid -> torch bf16 on the GPU (exact)."""
    return torch.from_numpy(np.ascontiguousarray(x_np)).cuda().to(torch.bfloat16)


def _run_prefill_case(h, nq, nkv, d, sl, n, pos0, max_seq, seed, attn_scale=1.0):
    rng = np.random.default_rng(seed)
    cfg = B.make_cfg(h, nq, nkv, d, sl, max_seq, dtype=B.TPI_BF16)
    oc = O.ShardCfg(h, nq, nkv, d, sl, max_seq)
    w = synth.make_layer_shard(rng, h, nq, nkv, d, sl)
    w["w_qkv"] = w["w_qkv"] * attn_scale
    wb = {k: (v if k.endswith("_norm") else synth.to_bf16_grid(v)) for k, v in w.items()}
    x = synth.to_bf16_grid(rng.standard_normal((n, h)).astype(np.float32))
    K = np.zeros((nkv, max_seq, d), np.float32); V = np.zeros_like(K)
    K[:, :pos0] = synth.to_bf16_grid(rng.standard_normal((nkv, pos0, d)).astype(np.float32))
    V[:, :pos0] = synth.to_bf16_grid(rng.standard_normal((nkv, pos0, d)).astype(np.float32))
    sentinel = 123.0
    K[:, pos0:] = sentinel; V[:, pos0:] = sentinel

    wt = {k: (torch.from_numpy(v).cuda() if k.endswith("_norm") else _bf16_t(v)) for k, v in wb.items()}
    Kt, Vt = _bf16_t(K), _bf16_t(V)
    xt = _bf16_t(x)
    nbytes = B.tpi_workspace_bytes(cfg, n)
    assert nbytes > 0
    ws = torch.full((nbytes // 4,), float("nan"), device="cuda")
    part = torch.empty((n, h), device="cuda")
    weights = B.make_weights(wt); kv = B.make_kv(Kt, Vt)
    B.tpi_shard_layer_prefill(cfg, weights, kv, pos0, n, B.TPI_PHASE_ATTN, xt, part, ws)
    torch.cuda.synchronize()
    got_attn = part.cpu().numpy().copy()
    Ko, Vo = K.copy(), V.copy()
    ref_attn = O.attn_block(oc, wb["attn_norm"], wb["w_qkv"], wb["w_o"], Ko, Vo, pos0, x)
    e = rel_err(got_attn, ref_attn)
    print(f"prefill h={h} nq={nq} nkv={nkv} d={d} n={n} pos0={pos0}: attention partial rel err {e:.2e}", flush=True)
    assert e <= BF16_TOL, f"attention partial rel err {e:.3e}"
    Kg, Vg = Kt.float().cpu().numpy(), Vt.float().cpu().numpy()
    for garr, before, after in ((Kg, K, Ko), (Vg, V, Vo)):
        changed = (garr != before).any(axis=2)
        expect = np.zeros_like(changed); expect[:, pos0:pos0 + n] = True
        assert np.array_equal(changed, expect), "cache slots outside pos0..pos0+n-1 touched, or some not written"
        assert rel_err(garr[:, pos0:pos0 + n], after[:, pos0:pos0 + n]) <= BF16_TOL
    # FFN phase on the same input
    B.tpi_shard_layer_prefill(cfg, weights, None, pos0, n, B.TPI_PHASE_FFN, xt, part, ws)
    torch.cuda.synchronize()
    ref_ffn = O.ffn_block(oc, wb["ffn_norm"], wb["w_gate"], wb["w_up"], wb["w_down"], x)
    e = rel_err(part.cpu().numpy(), ref_ffn)
    print(f"prefill h={h} sl={sl} n={n}: FFN partial rel err {e:.2e}", flush=True)
    assert e <= BF16_TOL, f"FFN partial rel err {e:.3e}"
    return got_attn, ref_attn


@pytest.mark.parametrize("h,nq,nkv,d,sl,n,pos0", [
    (256, 2, 2, 64, 344, 5, 0),        # tiny shard, a handful of tokens
    (256, 2, 2, 64, 344, 70, 0),       # more than one 64-token tile
    (256, 2, 2, 64, 344, 37, 29),      # non-empty cache in front
    (264, 4, 1, 128, 72, 129, 3),      # K not a multiple of 64, group of 4, ragged everything
    (512, 8, 1, 128, 256, 64, 0),      # the 70B head layout: 8 query heads on one KV head
    (128, 3, 3, 32, 64, 200, 0),       # small heads, several key tiles
    (192, 2, 1, 96, 64, 45, 2),        # head_dim 96: three 32-wide output tiles
    (96, 4, 2, 48, 40, 33, 0),         # head_dim not a multiple of 32: the vector-ALU attention
    (512, 16, 1, 64, 128, 150, 1),     # 16 query heads per KV head: a row tile covers two tokens
    (128, 4, 2, 32, 64, 1500, 37),     # long prompt on top of a cache: 48 key tiles, 12 rounds per wave
    (264, 2, 1, 64, 2776, 300, 0),     # gate|up with the activation in its epilogue (128-row tiles), ragged rows, units and K
    (128, 2, 1, 64, 8200, 40, 5),      # the same with 64-row tiles
    (8456, 2, 1, 64, 64, 9, 0),        # token rows longer than what the RMSNorm keeps in registers
])
def test_prefill_parity_small_shapes(h, nq, nkv, d, sl, n, pos0):
    _run_prefill_case(h, nq, nkv, d, sl, n, pos0, pos0 + n + 3, seed=h + n + pos0, attn_scale=4.0)


def _random_prefill_shapes(n, seed):
    """Seeded random shapes inside the documented limits of the bf16 path: every size a multiple of 8."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        d = int(rng.choice([8, 16, 32, 48, 64, 96, 128]))
        nkv = int(rng.integers(1, 3))
        G = int(rng.choice([1, 2, 3, 4, 8]))
        h = 8 * int(rng.integers(2, 80))
        sl = 8 * int(rng.integers(1, 90))
        n_tok = int(rng.integers(1, 200))
        pos0 = int(rng.choice([0, 0, int(rng.integers(0, 70))]))
        out.append((h, G * nkv, nkv, d, sl, n_tok, pos0))
    return out


@pytest.mark.parametrize("h,nq,nkv,d,sl,n,pos0", _random_prefill_shapes(12, 512))
def test_prefill_random_shapes(h, nq, nkv, d, sl, n, pos0):
    _run_prefill_case(h, nq, nkv, d, sl, n, pos0, pos0 + n + int(n % 3), seed=h + n + pos0 + d, attn_scale=4.0)


@pytest.mark.parametrize("h,nq,nkv,d,sl,n,pos0", [
    (264, 2, 1, 64, 2776, 300, 0),     # ragged rows, units and K on 128x256 tiles, gate|up with the activation fused
    (1096, 8, 1, 128, 520, 200, 3),    # output projection and down with 1096 columns: 4 full tiles and a ragged one
])
def test_prefill_parity_under_the_concurrency_hint(h, nq, nkv, d, sl, n, pos0):
    """With the hint that four prefill calls run side by side the GEMM plans take the wide tiles already at
    these sizes; the results must meet the same tolerance."""
    B.tpi_set_prefill_concurrency(4)
    try:
        _run_prefill_case(h, nq, nkv, d, sl, n, pos0, pos0 + n + 2, seed=h + n, attn_scale=4.0)
    finally:
        B.tpi_set_prefill_concurrency(1)


def test_prefill_single_token_and_last_slot():
    _run_prefill_case(256, 2, 2, 64, 344, 1, 0, 1, seed=1)
    _run_prefill_case(256, 2, 2, 64, 344, 1, 15, 16, seed=2)
    _run_prefill_case(256, 2, 2, 64, 344, 9, 7, 16, seed=3)


def test_prefill_8b_shaped_layer_one_shard():
    m = configs.LLAMA31_8B_TP4
    _run_prefill_case(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, 128, 0, 128, seed=8)


def test_prefill_70b_shaped_layer_one_shard_512_tokens():
    """The benchmark's prefill shape (70B-shaped 8-way shard): 512 prompt tokens, empty cache, one shard of one layer."""
    m = configs.LLAMA2_70B_TP8
    _run_prefill_case(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, 512, 0, 512, seed=70)


def test_prefill_partials_reduce_over_shards():
    """fp32 partials of 4 emulated shards star-reduced with the shortcut: bit-exact against the
    oracle's sequential fp32 reduce of the same GPU partials, and within tolerance of the oracle layer."""
    h, nq, nkv, d, sl, n, N = 256, 2, 1, 64, 128, 48, 4
    rng = np.random.default_rng(11)
    cfg = B.make_cfg(h, nq, nkv, d, sl, n, dtype=B.TPI_BF16)
    oc = O.ShardCfg(h, nq, nkv, d, sl, n)
    x = synth.to_bf16_grid(rng.standard_normal((n, h)).astype(np.float32))
    xt = _bf16_t(x)
    ws = torch.empty(B.tpi_workspace_bytes(cfg, n) // 4, device="cuda")
    parts, refs = [], []
    for r in range(N):
        w = synth.make_layer_shard(rng, h, nq, nkv, d, sl)
        wb = {k: (v if k.endswith("_norm") else synth.to_bf16_grid(v)) for k, v in w.items()}
        wt = {k: (torch.from_numpy(v).cuda() if k.endswith("_norm") else _bf16_t(v)) for k, v in wb.items()}
        Kt = torch.zeros((nkv, n, d), device="cuda", dtype=torch.bfloat16); Vt = torch.zeros_like(Kt)
        p = torch.empty((n, h), device="cuda")
        B.tpi_shard_layer_prefill(cfg, B.make_weights(wt), B.make_kv(Kt, Vt), 0, n, B.TPI_PHASE_ATTN, xt, p, ws)
        parts.append(p)
        K = np.zeros((nkv, n, d), np.float32); V = np.zeros_like(K)
        refs.append(O.attn_block(oc, wb["attn_norm"], wb["w_qkv"], wb["w_o"], K, V, 0, x))
    res = torch.from_numpy(x).cuda()
    out = torch.empty((n, h), device="cuda")
    B.tpi_star_reduce(parts, res, out)
    torch.cuda.synchronize()
    want_bits = O.reduce_seq_f32([p.cpu().numpy() for p in parts], x)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want_bits.view(np.uint32))
    assert rel_err(out.cpu().numpy(), O.reduce_f64(refs, x)) <= BF16_TOL


@pytest.mark.parametrize("h,nq,nkv,d,sl,n,pos0,N,shared_gains", [
    (512, 4, 1, 64, 1280, 300, 0, 4, False),      # wide tiles under the batch, gate|up fused
    (264, 2, 2, 32, 72, 70, 5, 3, False),         # ragged everything, small tiles, split-K QKV
    (192, 2, 1, 48, 64, 33, 0, 2, False),         # head_dim 48: the vector-ALU attention, one shard per launch
    (256, 2, 1, 64, 128, 40, 2, B.TPI_MAX_BATCH_SHARDS, False),
    (512, 4, 1, 64, 1280, 300, 0, 4, True),       # one replicated gain vector: the input is normalised once
    (264, 2, 2, 32, 72, 70, 5, 3, True),
])
def test_prefill_batched_call_matches_per_shard_calls_and_oracle(h, nq, nkv, d, sl, n, pos0, N, shared_gains):
    _batched_case(h, nq, nkv, d, sl, n, pos0, N, shared_gains)


def _batched_case(h, nq, nkv, d, sl, n, pos0, N, shared_gains=False):
    """tpi_shards_layer_prefill: all shards of a layer phase in one set of launches.  Per shard the result must
    agree with the single-shard call (the plans may differ: tolerance, not bits), the cache slots written must be
    the same set, and the first and the last shard are checked against the oracle.  shared_gains: every shard names
    the same norm gains (the norm is replicated on all devices, Sec. 3.1); the call then normalises once."""
    rng = np.random.default_rng(h + n + N)
    max_seq = pos0 + n + 1
    cfg = B.make_cfg(h, nq, nkv, d, sl, max_seq, dtype=B.TPI_BF16)
    oc = O.ShardCfg(h, nq, nkv, d, sl, max_seq)
    x = synth.to_bf16_grid(rng.standard_normal((n, h)).astype(np.float32))
    xt = _bf16_t(x)
    nws = B.tpi_workspace_bytes(cfg, n) // 4
    sh = []
    for r in range(N):
        w = synth.make_layer_shard(rng, h, nq, nkv, d, sl)
        wb = {k: (v if k.endswith("_norm") else synth.to_bf16_grid(v)) for k, v in w.items()}
        wt = {k: (torch.from_numpy(v).cuda() if k.endswith("_norm") else _bf16_t(v)) for k, v in wb.items()}
        if shared_gains and sh:
            for k in ("attn_norm", "ffn_norm"):
                wb[k] = sh[0]["wb"][k]; wt[k] = sh[0]["wt"][k]      # the same device tensor: the same pointer
        K = np.full((nkv, max_seq, d), 123.0, np.float32); V = K.copy()
        K[:, :pos0] = synth.to_bf16_grid(rng.standard_normal((nkv, pos0, d)).astype(np.float32))
        V[:, :pos0] = synth.to_bf16_grid(rng.standard_normal((nkv, pos0, d)).astype(np.float32))
        sh.append(dict(wb=wb, wt=wt, W=B.make_weights(wt), K=K, V=V,
                       Ka=_bf16_t(K), Va=_bf16_t(V), Kb=_bf16_t(K), Vb=_bf16_t(V),
                       wsa=torch.full((nws,), float("nan"), device="cuda"), wsb=torch.full((nws,), float("nan"), device="cuda")))
    for phase in (B.TPI_PHASE_ATTN, B.TPI_PHASE_FFN):
        pa = [torch.empty((n, h), device="cuda") for _ in range(N)]
        pb = [torch.empty((n, h), device="cuda") for _ in range(N)]
        attn = phase == B.TPI_PHASE_ATTN
        B.tpi_shards_layer_prefill(cfg, [s_["W"] for s_ in sh], [B.make_kv(s_["Ka"], s_["Va"]) for s_ in sh] if attn else None,
                                   pos0, n, phase, xt, pa, [s_["wsa"] for s_ in sh])
        for r, s_ in enumerate(sh):
            B.tpi_shard_layer_prefill(cfg, s_["W"], B.make_kv(s_["Kb"], s_["Vb"]) if attn else None, pos0, n, phase, xt,
                                      pb[r], s_["wsb"])
        torch.cuda.synchronize()
        for r, s_ in enumerate(sh):
            assert rel_err(pa[r].cpu().numpy(), pb[r].cpu().numpy()) <= 2e-3, f"shard {r}"
            if attn:
                ka, kb = s_["Ka"].float().cpu().numpy(), s_["Kb"].float().cpu().numpy()
                assert np.array_equal(ka != s_["K"], kb != s_["K"])          # the same slots written
                assert rel_err(ka[:, pos0:pos0 + n], kb[:, pos0:pos0 + n]) <= 1e-2
                assert rel_err(s_["Va"].float().cpu().numpy()[:, pos0:pos0 + n], s_["Vb"].float().cpu().numpy()[:, pos0:pos0 + n]) <= 1e-2
        for r in (0, N - 1):
            w0 = sh[r]["wb"]
            if attn:
                ref = O.attn_block(oc, w0["attn_norm"], w0["w_qkv"], w0["w_o"], sh[r]["K"].copy(), sh[r]["V"].copy(), pos0, x)
            else:
                ref = O.ffn_block(oc, w0["ffn_norm"], w0["w_gate"], w0["w_up"], w0["w_down"], x)
            assert rel_err(pa[r].cpu().numpy(), ref) <= BF16_TOL


def test_prefill_shards_on_two_streams_equal_one_stream_bitwise():
    """The emulated shards of a layer are independent between the reduces: dealt to two streams (each with a
    workspace of its own, joined by events before the reduce) they must give the bits of the one-stream run,
    under the same concurrency hint."""
    h, nq, nkv, d, sl, n, N = 512, 4, 1, 64, 1280, 300, 4
    rng = np.random.default_rng(31)
    cfg = B.make_cfg(h, nq, nkv, d, sl, n, dtype=B.TPI_BF16)
    xt = _bf16_t(synth.to_bf16_grid(rng.standard_normal((n, h)).astype(np.float32)))
    shards = []
    for r in range(N):
        w = synth.make_layer_shard(rng, h, nq, nkv, d, sl)
        wt = {k: (torch.from_numpy(v).cuda() if k.endswith("_norm") else _bf16_t(synth.to_bf16_grid(v))) for k, v in w.items()}
        Kt = torch.zeros((nkv, n, d), device="cuda", dtype=torch.bfloat16)
        shards.append((B.make_weights(wt), wt, Kt, torch.zeros_like(Kt)))
    nws = B.tpi_workspace_bytes(cfg, n) // 4

    def run(streams):
        main = torch.cuda.current_stream()
        wss = [torch.full((nws,), float("nan"), device="cuda") for _ in streams]
        outs = []
        for phase in (B.TPI_PHASE_ATTN, B.TPI_PHASE_FFN):
            parts = [torch.empty((n, h), device="cuda") for _ in range(N)]
            ev = torch.cuda.Event(); ev.record(main)
            for st in streams:
                st.wait_event(ev)
            for r, (W, _, Kt, Vt) in enumerate(shards):
                st = streams[r % len(streams)]
                B.tpi_shard_layer_prefill(cfg, W, B.make_kv(Kt, Vt) if phase == B.TPI_PHASE_ATTN else None, 0, n, phase,
                                          xt, parts[r], wss[r % len(streams)], stream=st)
            for st in streams:
                e2 = torch.cuda.Event(); e2.record(st); main.wait_event(e2)
            out = torch.empty((n, h), device="cuda")
            B.tpi_star_reduce(parts, None, out)
            outs.append(out)
        torch.cuda.synchronize()
        return outs

    B.tpi_set_prefill_concurrency(2)
    try:
        one = run([torch.cuda.current_stream()])
        two = run([torch.cuda.Stream(), torch.cuda.Stream()])
    finally:
        B.tpi_set_prefill_concurrency(1)
    for a, b in zip(one, two):
        assert torch.isfinite(a).all()
        assert torch.equal(a, b)


def test_star_reduce_bf16_copy_is_round_to_nearest_even():
    rng = np.random.default_rng(12)
    n, length = 5, 4099
    ps = [(rng.standard_normal(length) * 10 ** rng.uniform(-2, 2, length)).astype(np.float32) for _ in range(n)]
    res = rng.standard_normal(length).astype(np.float32)
    tp = [torch.from_numpy(p).cuda() for p in ps]
    out = torch.empty(length, device="cuda"); out2 = torch.empty(length, device="cuda")
    ob = torch.empty(length, device="cuda", dtype=torch.bfloat16)
    B.tpi_star_reduce_bf16(tp, torch.from_numpy(res).cuda(), out, ob)
    B.tpi_star_reduce(tp, torch.from_numpy(res).cuda(), out2)
    torch.cuda.synchronize()
    want = O.reduce_seq_f32(ps, res)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert torch.equal(out, out2)
    assert np.array_equal(ob.float().cpu().numpy(), synth.to_bf16_grid(want))
    # ties: 1 + 2^-8 lies midway between two bf16 values and must go to the even one (1.0);
    # 1 + 3*2^-8 midway again, goes up to 1 + 2^-6
    t = torch.tensor([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 0.0], device="cuda")
    ob4 = torch.empty(4, device="cuda", dtype=torch.bfloat16); o4 = torch.empty(4, device="cuda")
    B.tpi_star_reduce_bf16([t], None, o4, ob4); torch.cuda.synchronize()
    assert ob4.float().tolist() == [1.0, 1.0 + 2.0 ** -6, -1.0, 0.0]


@pytest.mark.parametrize("h,nq,nkv,d,sl,n,N,L,batched", [
    (256, 2, 1, 64, 344, 70, 2, 3, False),
    (256, 2, 1, 64, 344, 70, 2, 3, True),
    (1024, 8, 1, 128, 1792, 512, 2, 8, False),     # an eighth of the 70B-shaped shard's width, the benchmark's prompt length
    (1024, 8, 1, 128, 1792, 512, 2, 8, True),
])
def test_prefill_stack_teacher_forced_and_free_running(h, nq, nkv, d, sl, n, N, L, batched):
    """A prompt through a stack the way bench.py chains the calls (attention phase -> reduce with the bf16 copy ->
    FFN phase -> reduce), with one call per shard or all shards per call (batched).  The oracle follows the same
    interface: fp32 hidden state as the shortcut, its bf16 rounding as the next block's input.  Every layer is
    checked teacher-forced (device layer run from the oracle's input) and the whole chain free-running: both
    arrangements must stay inside the bf16 tolerance of the oracle over the whole stack, whatever they differ by
    from each other."""
    rng = np.random.default_rng(21)
    cfg = B.make_cfg(h, nq, nkv, d, sl, n, dtype=B.TPI_BF16)
    oc = O.ShardCfg(h, nq, nkv, d, sl, n)
    ws = torch.empty(B.tpi_workspace_bytes(cfg, n) // 4, device="cuda")
    wsb = [torch.empty(B.tpi_workspace_bytes(cfg, n) // 4, device="cuda") for _ in range(N)]
    stack = []
    for l in range(L):
        row = []
        for r in range(N):
            w = synth.make_layer_shard(rng, h, nq, nkv, d, sl)
            wb = {k: (v if k.endswith("_norm") else synth.to_bf16_grid(v)) for k, v in w.items()}
            wt = {k: (torch.from_numpy(v).cuda() if k.endswith("_norm") else _bf16_t(v)) for k, v in wb.items()}
            row.append((wb, wt, B.make_weights(wt)))
        stack.append(row)

    def gpu_layer(l, x32_t):
        x16 = x32_t.to(torch.bfloat16)
        parts = [torch.empty((n, h), device="cuda") for _ in range(N)]
        caches = [(torch.zeros((nkv, n, d), device="cuda", dtype=torch.bfloat16),
                   torch.zeros((nkv, n, d), device="cuda", dtype=torch.bfloat16)) for _ in range(N)]
        W = [stack[l][r][2] for r in range(N)]
        if batched:
            B.tpi_shards_layer_prefill(cfg, W, [B.make_kv(Kt, Vt) for Kt, Vt in caches], 0, n, B.TPI_PHASE_ATTN, x16, parts, wsb)
        else:
            for r in range(N):
                B.tpi_shard_layer_prefill(cfg, W[r], B.make_kv(*caches[r]), 0, n, B.TPI_PHASE_ATTN, x16, parts[r], ws)
        a32 = torch.empty_like(x32_t); a16 = torch.empty_like(x16)
        B.tpi_star_reduce_bf16(parts, x32_t, a32, a16)
        if batched:
            B.tpi_shards_layer_prefill(cfg, W, None, 0, n, B.TPI_PHASE_FFN, a16, parts, wsb)
        else:
            for r in range(N):
                B.tpi_shard_layer_prefill(cfg, W[r], None, 0, n, B.TPI_PHASE_FFN, a16, parts[r], ws)
        o32 = torch.empty_like(x32_t); o16 = torch.empty_like(x16)
        B.tpi_star_reduce_bf16(parts, a32, o32, o16)
        torch.cuda.synchronize()
        return a32, o32

    def oracle_layer(l, x32):
        x16 = synth.to_bf16_grid(x32)
        pa = []
        for r in range(N):
            wb = stack[l][r][0]
            K = np.zeros((nkv, n, d), np.float32); V = np.zeros_like(K)
            pa.append(O.attn_block(oc, wb["attn_norm"], wb["w_qkv"], wb["w_o"], K, V, 0, x16))
        a32 = O.reduce_f64(pa, x32).astype(np.float32)
        a16 = synth.to_bf16_grid(a32)
        pf = [O.ffn_block(oc, stack[l][r][0]["ffn_norm"], stack[l][r][0]["w_gate"], stack[l][r][0]["w_up"],
                          stack[l][r][0]["w_down"], a16) for r in range(N)]
        return a32, O.reduce_f64(pf, a32).astype(np.float32)

    x0 = synth.to_bf16_grid(rng.standard_normal((n, h)).astype(np.float32))
    x_orc, x_gpu = x0, torch.from_numpy(x0).cuda()
    worst_tf = worst_free = 0.0
    for l in range(L):
        ra, ro = oracle_layer(l, x_orc)
        ta, to = gpu_layer(l, torch.from_numpy(x_orc).cuda())                  # teacher-forced
        worst_tf = max(worst_tf, rel_err(ta.cpu().numpy(), ra), rel_err(to.cpu().numpy(), ro))
        fa, fo = gpu_layer(l, x_gpu)                                           # free-running
        worst_free = max(worst_free, rel_err(fa.cpu().numpy(), ra), rel_err(fo.cpu().numpy(), ro))
        x_orc, x_gpu = ro, fo
    print(f"prefill stack h={h} n={n}, {L} layers x {N} shards, {'all shards per call' if batched else 'one shard per call'}: "
          f"worst rel err vs oracle teacher-forced {worst_tf:.2e}, free-running {worst_free:.2e}", flush=True)
    assert worst_tf <= BF16_TOL
    assert worst_free <= BF16_TOL


def test_prefill_gate_up_divided_between_wide_and_narrow_tiles():
    """When the wide gate|up tiles would end with a nearly empty last round of the compute units, the hidden units
    are divided between a launch of wide tiles and one of 128-column tiles.  With the hint at its maximum the call
    counts on 16 compute units, which brings that division to small shapes: 1120 units = 1024 on wide tiles + 96,
    and, for two shards per call, 616 = 512 + 104 (the last tile ragged in both)."""
    B.tpi_set_prefill_concurrency(B.TPI_MAX_BATCH_SHARDS)
    try:
        _run_prefill_case(320, 2, 1, 64, 1120, 200, 0, 202, seed=5, attn_scale=4.0)
        _batched_case(320, 2, 1, 64, 616, 200, 0, 2)
    finally:
        B.tpi_set_prefill_concurrency(1)


@pytest.mark.parametrize("steps", [1, 2, 3, 4, 5])
def test_prefill_direct_to_lds_tiles_with_few_k_steps(steps):
    """The GEMM variant that loads its tiles straight into LDS runs its K loop in rounds of three steps with the
    one or two left over after it.  Output projection (K = n_q * 64) and down projection (K = ffn) with 1..5
    K-steps of 64, on 128x128 tiles (the hint makes the planner keep them at this size)."""
    B.tpi_set_prefill_concurrency(B.TPI_MAX_BATCH_SHARDS)
    try:
        _run_prefill_case(512, steps, 1, 64, 64 * steps, 130, 0, 131, seed=40 + steps, attn_scale=4.0)
    finally:
        B.tpi_set_prefill_concurrency(1)


@pytest.mark.parametrize("h", [512, 576])
def test_prefill_two_stage_direct_tiles(h):
    """A 128x128-tile GEMM with at least two workgroups per compute unit takes the two-stage variant of the
    direct-to-LDS loop (two workgroups resident per compute unit).  QKV with 2048 output rows on 130 tokens is
    32 tiles; under the maximum hint the call counts on 16 compute units.  8 and 9 K-steps: an even count and
    one left over."""
    B.tpi_set_prefill_concurrency(B.TPI_MAX_BATCH_SHARDS)
    try:
        _run_prefill_case(h, 24, 4, 64, 256, 130, 0, 131, seed=h, attn_scale=4.0)
    finally:
        B.tpi_set_prefill_concurrency(1)


@pytest.mark.parametrize("h,n", [(2048, 300), (2112, 257)])
def test_prefill_256x256_tiles_at_a_small_size(h, n):
    """Products whose 256x256 tiles fill the compute units the call counts on take the eight-wave 256x256 tile (two
    LDS stages, every wave all four slices of a K-step).  Under the maximum hint that is 16 compute units, which
    brings the choice to a small shape: 960 hidden units = 8 column tiles of gate|up (the last one half empty) on 2
    row tiles (the second with 44 rows, or with 1), the down projection with 15 K-steps (one left over after the
    rounds of two), the output projection with 8, and the QKV product (1024 columns) split 2-way along K over 8
    tiles: 16 + 16 K-steps at h = 2048, 17 + 16 at h = 2112."""
    B.tpi_set_prefill_concurrency(B.TPI_MAX_BATCH_SHARDS)
    try:
        _run_prefill_case(h, 8, 4, 64, 960, n, 0, n + 1, seed=h + n)
    finally:
        B.tpi_set_prefill_concurrency(1)


@pytest.mark.parametrize("steps", [1, 2, 3, 4, 5])
def test_prefill_256x256_tiles_with_few_k_steps(steps):
    """The two-stage loop of the 256x256 tile with 1..5 K-steps of 64 (rounds of two steps, one left over, and the
    requests that repeat the last step): output projection (K = n_q * 64) and down projection (K = ffn) onto 2048
    columns, 300 tokens, under the maximum hint (16 tiles = the 16 compute units the call counts on)."""
    B.tpi_set_prefill_concurrency(B.TPI_MAX_BATCH_SHARDS)
    try:
        _run_prefill_case(2048, steps, 1, 64, 64 * steps, 300, 0, 301, seed=70 + steps)
    finally:
        B.tpi_set_prefill_concurrency(1)


def test_prefill_gate_up_divided_between_256_and_192_column_tiles():
    """When the 256x256 tiles of gate|up end with a ragged round whose units make exactly one round of 256x192
    tiles (96 units each; gate sums in the left wave column, up sums in the right one, exchanged through LDS before
    the activation), the launch is divided.  Under the maximum hint (16 compute units): 300 tokens = 2 row tiles,
    1720 units = 14 column tiles = 28 tiles; the first 8 column tiles make one whole round, the other 696 units
    make 8 tiles of 96 (the last with 24 units) on the 2 row tiles = the second round."""
    B.tpi_set_prefill_concurrency(B.TPI_MAX_BATCH_SHARDS)
    try:
        _run_prefill_case(512, 4, 2, 64, 1720, 300, 0, 301, seed=1720)
    finally:
        B.tpi_set_prefill_concurrency(1)


@pytest.mark.parametrize("h,nq,nkv,d,sl,n,pos0", [
    (256, 16, 4, 64, 64, 300, 5),      # 4 heads per KV head, non-empty cache, 1200 rows per KV head: a ragged last block
    (512, 8, 1, 128, 64, 530, 0),      # head_dim 128, 8 heads on one KV head, 17 key tiles (rounds of three and two left over)
    (256, 4, 4, 64, 64, 1030, 0),      # one head per KV head
    (256, 8, 2, 64, 64, 260, 33),      # keys before the prompt: every row sees at least two tiles
])
def test_prefill_attention_with_tiles_shared_by_128_rows(h, nq, nkv, d, sl, n, pos0):
    """Prompts with at least one 128-row workgroup per compute unit take the attention kernel that brings each
    key / value tile into LDS once per 128 rows and reads V through the transposing LDS load.  The maximum hint
    (16 compute units to count on) brings that choice to these sizes."""
    B.tpi_set_prefill_concurrency(B.TPI_MAX_BATCH_SHARDS)
    try:
        _run_prefill_case(h, nq, nkv, d, sl, n, pos0, pos0 + n + 1, seed=h + n + d, attn_scale=4.0)
    finally:
        B.tpi_set_prefill_concurrency(1)



@pytest.mark.parametrize("n", [512, 333])
def test_prefill_70b_shaped_8_shards_in_one_call(n):
    """What the benchmark's prefill leg times, at its real size: tpi_shards_layer_prefill with all 8 shards of a
    70B-shaped layer and the prompt's tokens in ONE call per phase (256x256 tiles for every product, the 3-way split
    of the QKV product over them and the shared-tile attention all at once); 512 tokens as in the benchmark, and 333,
    where the second row tile of every product is ragged (77 of 256 rows).  Two of the shards are checked element
    by element against the oracle (about 10 s of CPU each), every shard's cache must have exactly slots 0..n-1
    written, and all shards must agree with their own single-shard call within the bf16 tolerance."""
    m = configs.LLAMA2_70B_TP8
    h, nq, nkv, d, sl, N = m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, m.n_shards
    pos0, max_seq = 0, n + 8
    cfg = B.make_cfg(h, nq, nkv, d, sl, max_seq, dtype=B.TPI_BF16)
    oc = O.ShardCfg(h, nq, nkv, d, sl, max_seq)
    gen = torch.Generator(device="cuda"); gen.manual_seed(512)
    shapes = synth.shard_tensor_shapes(h, nq, nkv, d, sl)
    xt = torch.randn((n, h), generator=gen, device="cuda").to(torch.bfloat16)
    nws = B.tpi_workspace_bytes(cfg, n) // 4
    sentinel = 123.0
    sh = []
    for r in range(N):
        wt = {}
        for name, shp in shapes.items():
            t = torch.randn(shp, generator=gen, device="cuda", dtype=torch.float32) * synth.WEIGHT_STD
            wt[name] = (t + 1.0) if name.endswith("_norm") else t.to(torch.bfloat16)
        K = torch.full((nkv, max_seq, d), sentinel, device="cuda", dtype=torch.bfloat16); V = K.clone()
        sh.append(dict(wt=wt, W=B.make_weights(wt), K=K, V=V, ws=torch.full((nws,), float("nan"), device="cuda")))
    checked = (0, N - 1)
    x = xt.float().cpu().numpy()
    for phase in (B.TPI_PHASE_ATTN, B.TPI_PHASE_FFN):
        attn = phase == B.TPI_PHASE_ATTN
        parts = [torch.full((n, h), float("nan"), device="cuda") for _ in range(N)]
        B.tpi_shards_layer_prefill(cfg, [s_["W"] for s_ in sh], [B.make_kv(s_["K"], s_["V"]) for s_ in sh] if attn else None,
                                   pos0, n, phase, xt, parts, [s_["ws"] for s_ in sh])
        torch.cuda.synchronize()
        if attn:
            for r, s_ in enumerate(sh):
                for t in (s_["K"], s_["V"]):
                    changed = (t.float() != sentinel).any(dim=2).cpu().numpy()
                    expect = np.zeros_like(changed); expect[:, pos0:pos0 + n] = True
                    assert np.array_equal(changed, expect), f"shard {r}: cache slots outside 0..{n - 1} touched, or some not written"
        # every shard against its own single-shard call (other plans, other attention kernel: tolerance, not bits)
        one = torch.empty((n, h), device="cuda")
        ws1 = torch.full((nws,), float("nan"), device="cuda")
        for r, s_ in enumerate(sh):
            K1 = torch.full_like(s_["K"], sentinel); V1 = K1.clone()
            B.tpi_shard_layer_prefill(cfg, s_["W"], B.make_kv(K1, V1) if attn else None, pos0, n, phase, xt, one, ws1)
            torch.cuda.synchronize()
            e = rel_err(parts[r].cpu().numpy(), one.cpu().numpy())
            assert e <= 1e-2, f"shard {r}, phase {phase}: batched vs single call rel err {e:.3e}"
        for r in checked:
            w = {k: v.float().cpu().numpy() for k, v in sh[r]["wt"].items()}
            if attn:
                Ko = np.zeros((nkv, max_seq, d), np.float32); Vo = np.zeros_like(Ko)
                ref = O.attn_block(oc, w["attn_norm"], w["w_qkv"], w["w_o"], Ko, Vo, pos0, x)
                Kg, Vg = sh[r]["K"].float().cpu().numpy(), sh[r]["V"].float().cpu().numpy()
                assert rel_err(Kg[:, :n], Ko[:, :n]) <= BF16_TOL and rel_err(Vg[:, :n], Vo[:, :n]) <= BF16_TOL
            else:
                ref = O.ffn_block(oc, w["ffn_norm"], w["w_gate"], w["w_up"], w["w_down"], x)
            e = rel_err(parts[r].cpu().numpy(), ref)
            print(f"70B-shaped prefill, 8 shards x {n} tokens in one call, shard {r}, phase {phase}: rel err {e:.2e}", flush=True)
            assert e <= BF16_TOL, f"shard {r}, phase {phase}: rel err {e:.3e}"


def test_prefill_then_decode_on_one_cache():
    """Sec. 3.1: the cache a device fills for its heads during the prompt serves every later token.  A prompt goes
    through the bf16 prefill, tpi_kv_widen carries the cache over to the fp32 cache of the decode entry points
    (exactly, and nothing beyond the prompt's slots), and the next token's attention phase on that cache agrees
    with the oracle, which ran the prompt and the token on one cache of its own."""
    h, nq, nkv, d, sl, n, max_seq = 256, 4, 2, 64, 344, 37, 48
    rng = np.random.default_rng(21)
    cfg16 = B.make_cfg(h, nq, nkv, d, sl, max_seq, dtype=B.TPI_BF16)
    cfg32 = B.make_cfg(h, nq, nkv, d, sl, max_seq + 4)                     # the decode cache may be longer
    oc = O.ShardCfg(h, nq, nkv, d, sl, max_seq + 4)
    w = synth.make_layer_shard(rng, h, nq, nkv, d, sl)
    wb = {k: (v if k.endswith("_norm") else synth.to_bf16_grid(v)) for k, v in w.items()}
    x = synth.to_bf16_grid(rng.standard_normal((n, h)).astype(np.float32))
    x_new = rng.standard_normal(h).astype(np.float32)
    # prompt
    wt16 = {k: (torch.from_numpy(v).cuda() if k.endswith("_norm") else _bf16_t(v)) for k, v in wb.items()}
    K16 = torch.zeros((nkv, max_seq, d), device="cuda", dtype=torch.bfloat16); V16 = torch.zeros_like(K16)
    part = torch.empty((n, h), device="cuda")
    ws16 = torch.empty(B.tpi_workspace_bytes(cfg16, n) // 4, device="cuda")
    B.tpi_shard_layer_prefill(cfg16, B.make_weights(wt16), B.make_kv(K16, V16), 0, n, B.TPI_PHASE_ATTN, _bf16_t(x), part, ws16)
    # carry the cache over
    sentinel = 7.5
    K32 = torch.full((nkv, max_seq + 4, d), sentinel, device="cuda"); V32 = torch.full_like(K32, sentinel)
    B.tpi_kv_widen(K16, V16, K32, V32, n)
    torch.cuda.synchronize()
    assert torch.equal(K32[:, :n], K16[:, :n].float()) and torch.equal(V32[:, :n], V16[:, :n].float())
    assert bool((K32[:, n:] == sentinel).all()) and bool((V32[:, n:] == sentinel).all())
    # the next token
    wt32 = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in wb.items()}
    out = torch.empty(h, device="cuda")
    ws32 = torch.empty(B.tpi_workspace_bytes(cfg32, 1) // 4, device="cuda")
    B.tpi_shard_layer_decode(cfg32, B.make_weights(wt32), B.make_kv(K32, V32), n, B.TPI_PHASE_ATTN,
                             torch.from_numpy(x_new).cuda(), out, ws32)
    torch.cuda.synchronize()
    Ko = np.zeros((nkv, max_seq + 4, d), np.float32); Vo = np.zeros_like(Ko)
    O.attn_block(oc, wb["attn_norm"], wb["w_qkv"], wb["w_o"], Ko, Vo, 0, x)
    ref = O.attn_block(oc, wb["attn_norm"], wb["w_qkv"], wb["w_o"], Ko, Vo, n, x_new)
    e = rel_err(out.cpu().numpy(), ref)
    assert e <= BF16_TOL, f"token after the prompt: rel err {e:.3e}"
    assert rel_err(K32[:, n].cpu().numpy(), Ko[:, n]) <= 1e-4       # the new slot is an fp32 one


def test_kv_widen_argument_errors():
    K16 = torch.zeros((2, 8, 64), device="cuda", dtype=torch.bfloat16)
    K32 = torch.zeros((2, 6, 64), device="cuda")
    with pytest.raises(B.TpiError) as ei:
        B.tpi_kv_widen(K16, K16, K32, K32, 7)          # more slots than the fp32 cache has
    assert ei.value.code == B.TPI_EINVAL
    B.tpi_kv_widen(K16, K16, K32, K32, 0)              # nothing to do is fine
