#!/usr/bin/env python3
"""Decode benchmark of the TPI-LLM shard path on one MI355X.

One step = one token through the whole layer stack: for every layer, the
attention phase of all N emulated shards, the fixed-order star reduce with the
shortcut, the FFN phase of all shards, and the second star reduce.  Default
workload: Llama-2-70B-shaped stack (80 layers, hidden 8192, 64 query / 8 KV
heads of 128, FFN 28672) cut 8 ways, every shard's fp32 weights resident in
HBM (273.85 GB), batch 1, KV length 1024, synthetic seeded data.

Prints ONE JSON line.  `value` is ms per token for the whole emulated job (all
8 shards on this one GPU); `one_shard` gives the same token for a single
device's shard (what one TPI-LLM device executes), with the 8-way reduce still
running on 7 pre-filled peer partials.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama2-70b-shaped-tp8",
                    choices=["llama2-70b-shaped-tp8", "llama3.1-8b-shaped-tp4", "tiny"])
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging)")
    ap.add_argument("--kv-len", type=int, default=0, help="tokens already cached (default 1024 / 512 / 16)")
    ap.add_argument("--mode", default="both", choices=["both", "all", "one"],
                    help="all: only the 8-shard emulated job; one: only one device's shard; both (default)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference row for rocprofv3 --pmc byte counters)")
    ap.add_argument("--no-window", action="store_true", help="skip the windowed-weights leg")
    ap.add_argument("--window-layers", type=int, default=4)
    ap.add_argument("--window-steps", type=int, default=3)
    ap.add_argument("--no-fused", action="store_true", help="skip the reduce-folded-into-phase leg")
    ap.add_argument("--separate-reduce", action="store_true",
                    help="time the all-shards step with separate star-reduce launches (default: folded into the "
                         "row-parallel stage, bitwise the same result)")
    ap.add_argument("--no-prefill", action="store_true", help="skip the bf16 prefill leg")
    ap.add_argument("--prefill-tokens", type=int, default=512)
    ap.add_argument("--prefill-steps", type=int, default=3)
    ap.add_argument("--no-prefill-batched", action="store_true", help="skip the all-shards-per-call prefill")
    ap.add_argument("--prefill-streams", type=int, default=2,
                    help="also time the prompt with the emulated shards dealt to this many streams (<= 1: skip)")
    ap.add_argument("--no-token-ends", action="store_true", help="skip embedding / task head / token choice")
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--no-window-files", action="store_true", help="skip the file-tier window (weights read from files)")
    ap.add_argument("--window-file-layers", type=int, default=16)
    ap.add_argument("--window-file-readers", type=int, default=4)
    ap.add_argument("--no-window-blocks", action="store_true",
                    help="skip the block-granular window variants (attention / FFN blocks, FFN retention)")
    ap.add_argument("--window-retain-every", type=int, default=2,
                    help="T of the retention variant: the FFN block of every T-th layer stays resident")
    ap.add_argument("--no-window-prefill", action="store_true",
                    help="skip the windowed long-prompt prefill (the point where the copies can hide)")
    ap.add_argument("--window-prefill-tokens", type=int, default=24576)
    ap.add_argument("--window-prefill-layers", type=int, default=16)
    ap.add_argument("--no-handover-probe", action="store_true",
                    help="skip the measurement of what a hand-over between dependent streaming stages costs")
    ap.add_argument("--no-gemm-probe", action="store_true",
                    help="skip the measurement of what paces the K loop of the prefill's 256x256 GEMM tile")
    ap.add_argument("--no-config2", action="store_true",
                    help="skip the short leg on the other configuration of the north star (8B-shaped, 4 shards x 32 layers)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle timing")
    ap.add_argument("--seed", type=int, default=0)
    return ap.parse_args()


def blob_layout(m):
    """Offsets (floats) of the seven tensors inside one layer-shard blob."""
    from paper_2410_00531_amd import synth
    shapes = synth.shard_tensor_shapes(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local)
    off, out = 0, {}
    for name in synth.TENSOR_ORDER:
        n = 1
        for s in shapes[name]:
            n *= s
        out[name] = (off, shapes[name], n)
        off += n
    return out, off


def stage_bytes(m, n_shards, pos):
    """Algorithmic bytes one launch of each stage moves (fp32): the weights it
    must read once, its input and output vectors, and the KV rows."""
    h, d, sl = m.hidden, m.head_dim, m.ffn_local
    dq, dkv = m.nq_local * d, m.nkv_local * d
    f = 4
    per = {
        "qkv": ((dq + 2 * dkv) * h + 2 * h + dq + 2 * dkv) * f,
        "attn": (2 * dkv * (pos + 1) + 2 * dq) * f,
        "oproj": (h * dq + dq + h) * f,
        "gate_up": (2 * sl * h + 2 * h + sl) * f,
        "down": (h * sl + sl + h) * f,
    }
    return {k: v * n_shards for k, v in per.items()}


def token_bytes(m, n_shards, n_reduce, n_layers, pos):
    sb = stage_bytes(m, n_shards, pos)
    reduce_b = (n_reduce + 2) * m.hidden * 4          # N partials + shortcut read, one write
    return n_layers * (sum(sb.values()) + 2 * reduce_b)


def token_ends_leg(args, m, ms_token):
    """The master's share outside the layers (Alg. 1 Preprocess / Postprocess): embedding row, final norm +
    task head (a streaming GEMV over vocab x hidden fp32), softmax + token choice.  Vocabulary 32000 as in
    the Llama 2 models of the paper's model table."""
    import torch

    from paper_2410_00531_amd import binding as B
    dev = torch.device("cuda:0")
    vocab, h = args.vocab, m.hidden
    gen = torch.Generator(device=dev); gen.manual_seed(args.seed + 3)
    w_head = torch.empty((vocab, h), dtype=torch.float32, device=dev).normal_(0.0, 0.02, generator=gen)
    norm = torch.empty(h, dtype=torch.float32, device=dev).normal_(1.0, 0.02, generator=gen)
    x = torch.randn(h, generator=gen, device=dev)
    logits = torch.empty(vocab, dtype=torch.float32, device=dev)
    tok = torch.zeros(1, dtype=torch.int32, device=dev)
    hx = torch.empty(h, dtype=torch.float32, device=dev)

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    us_head = timed(lambda: B.tpi_lm_head(norm, w_head, x, logits, m.rms_eps))
    us_pick = timed(lambda: B.tpi_next_token(logits, 0.5, tok))
    us_emb = timed(lambda: B.tpi_embed_token(w_head, 17, hx))      # any [vocab][hidden] table serves as W_emb here
    head_bytes = (vocab * h + 2 * h + vocab) * 4
    ends_ms = (us_head + us_pick + us_emb) / 1e3
    return {
        "vocab": vocab, "lm_head_us": round(us_head, 1), "lm_head_gb": round(head_bytes / 1e9, 3),
        "lm_head_gbps": round(head_bytes / (us_head * 1e-6) / 1e9, 1),
        "lm_head_frac_of_peak": round(head_bytes / (us_head * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "next_token_us": round(us_pick, 1), "embed_us": round(us_emb, 1),
        "ms_per_token_with_ends": round(ms_token + ends_ms, 4), "token": int(tok.item()),
    }


def window_leg(args, m, L, N, blobs, layout, blob_floats, cfg, KV_one, P_all, P_one, WS_one, h0, h_a, h_b, h_attn,
               pos0, ms_resident):
    """Shard 0 again, but its layer blobs live in pinned host memory and pass through a ring of
    --window-layers HBM slots, refilled by async copies while earlier layers compute."""
    import torch

    from paper_2410_00531_amd import binding as B
    from paper_2410_00531_amd import synth
    dev = h0.device
    Wn = min(args.window_layers, L)
    nbytes = blob_floats * 4
    host = []
    for l in range(L):
        hb = torch.empty(blob_floats, dtype=torch.float32, pin_memory=True)
        hb.copy_(blobs[l][0])
        host.append(hb)
    slots = torch.empty(Wn * blob_floats, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    # practical peak of the link: plain pinned host-to-device copies of one blob
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 8
    slots[:blob_floats].copy_(host[0], non_blocking=True)
    e0.record()
    for i in range(reps):
        slots[:blob_floats].copy_(host[i % L], non_blocking=True)
    e1.record(); torch.cuda.synchronize()
    link_gbps = reps * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9

    lib = B.lib()
    stream = torch.cuda.current_stream().cuda_stream
    cfg_p = C.byref(cfg)
    by_ptr = {}
    for s_i in range(Wn):
        w = (B.tpi_layer_weights * 1)()
        base = slots.data_ptr() + s_i * nbytes
        for name in synth.TENSOR_ORDER:
            setattr(w[0], name, base + layout[name][0] * 4)
        by_ptr[base] = w
    win = B.Window(host, slots, Wn, nbytes)
    win.calibrate()
    for l in range(Wn):
        win.prefetch(l)
    nxt = [Wn]

    def check(rc):
        if rc != 0:
            raise RuntimeError(B.tpi_last_error())

    def token(pos):
        src, dst = h0, h_a
        for l in range(L):
            w = by_ptr[win.acquire(l)]
            check(lib.tpi_shards_layer_decode(cfg_p, 1, w, KV_one[l], pos, B.TPI_PHASE_ATTN, src.data_ptr(),
                                              P_one, WS_one, stream))
            check(lib.tpi_star_reduce(P_all, N, m.hidden, src.data_ptr(), h_attn.data_ptr(), stream))
            check(lib.tpi_shards_layer_decode(cfg_p, 1, w, None, pos, B.TPI_PHASE_FFN, h_attn.data_ptr(),
                                              P_one, WS_one, stream))
            check(lib.tpi_star_reduce(P_all, N, m.hidden, h_attn.data_ptr(), dst.data_ptr(), stream))
            win.release(l)
            win.prefetch(nxt[0] % L)            # slides on into the next token's layers
            nxt[0] += 1
            src, dst = dst, (h_b if dst is h_a else h_a)
        return src

    token(pos0)                                  # warm-up token (the first window was preloaded)
    # only the compute stream: a device-wide wait would also let the copies of the next token's first layers
    # finish before the clock starts, and the timed tokens would get them for free
    torch.cuda.current_stream().synchronize()
    t = time.perf_counter()
    for i in range(args.window_steps):
        out = token(pos0 + 1 + i)
    torch.cuda.current_stream().synchronize()
    ms = (time.perf_counter() - t) * 1e3 / args.window_steps
    finite = bool(torch.isfinite(out).all().item())
    win.destroy()
    copy_ms = L * nbytes / (link_gbps * 1e9) * 1e3
    res = {
        "workload": f"{m.name}-windowed-decode-one-shard", "window_layers": Wn, "steps": args.window_steps,
        "ms_per_token": round(ms, 2), "tokens_per_s": round(1e3 / ms, 3),
        "h2d_gb_per_token": round(L * nbytes / 1e9, 3), "pcie_gbps": round(L * nbytes / (ms * 1e-3) / 1e9, 2),
        "link_peak_gbps_plain_copy": round(link_gbps, 2),
        "pcie_frac_of_plain_copy": round(L * nbytes / (ms * 1e-3) / 1e9 / link_gbps, 4),
        "copy_ms_per_token_at_link_peak": round(copy_ms, 2), "resident_ms_per_token": round(ms_resident, 3),
        "hidden_fraction": round(max(0.0, 1.0 - (ms - ms_resident) / copy_ms), 4),
        "compute_over_copy": round(ms_resident / copy_ms, 4), "output_finite": finite,
    }
    if not args.no_window_files:
        res["file_tier"] = window_files_variant(args, m, L, N, blobs, layout, cfg, KV_one, P_all, P_one, WS_one, h0, h_a,
                                                h_b, h_attn, pos0, link_gbps)
    if not args.no_window_blocks and Wn >= 2:
        res["block_granular"] = [
            window_blocks_variant(args, m, L, N, blobs, host, layout, cfg, KV_one, P_all, P_one, WS_one, h0, h_a, h_b,
                                  h_attn, pos0, link_gbps, T)
            for T in (0, args.window_retain_every)]
    return res


def window_files_variant(args, m, L, N, blobs, layout, cfg, KV_one, P_all, P_one, WS_one, h0, h_a, h_b, h_attn, pos0,
                         link_gbps):
    """The paper's source tier: the layer blobs of shard 0 are files, a loader thread reads them into two
    pinned staging buffers and forwards them into the HBM slots.  --window-file-layers layers per token
    (a token over all 80 would only repeat the same steady state); 8 distinct files, layer l uses file l % 8.
    The files have just been written, so they are read through the page cache: the figure is the rate of
    the loader path (pread into pinned memory, then the copy over the link), not of a disk."""
    import shutil
    import tempfile

    import torch

    from paper_2410_00531_amd import binding as B
    from paper_2410_00531_amd import synth
    dev = h0.device
    Lf = min(args.window_file_layers, L)
    Wn = min(args.window_layers, Lf)
    D = min(8, Lf)
    nfl = blobs[0][0].numel()
    nbytes = nfl * 4
    tmp = tempfile.mkdtemp(prefix="tpi_blobs_")
    try:
        paths = []
        for i in range(D):
            path = os.path.join(tmp, f"layer{i}.bin")
            blobs[i][0].cpu().numpy().tofile(path)
            paths.append(path)
        slots = torch.empty(Wn * nfl, dtype=torch.float32, device=dev)
        by_ptr = {}
        for s_i in range(Wn):
            w = (B.tpi_layer_weights * 1)()
            base = slots.data_ptr() + s_i * nbytes
            for name in synth.TENSOR_ORDER:
                setattr(w[0], name, base + layout[name][0] * 4)
            by_ptr[base] = w
        win = B.Window.from_files([(paths[l % D], 0, nbytes, 0, None) for l in range(Lf)], [(slots, nbytes, Wn)],
                                  n_staging=2, n_readers=args.window_file_readers)
        lib = B.lib()
        stream = torch.cuda.current_stream().cuda_stream
        cfg_p = C.byref(cfg)
        for l in range(Wn):
            win.prefetch(l)
        nxt = [Wn]

        def check(rc):
            if rc != 0:
                raise RuntimeError(B.tpi_last_error())

        def token(pos):
            src, dst = h0, h_a
            for l in range(Lf):
                w = by_ptr[win.acquire(l)]
                check(lib.tpi_shards_layer_decode(cfg_p, 1, w, KV_one[l], pos, B.TPI_PHASE_ATTN, src.data_ptr(),
                                                  P_one, WS_one, stream))
                check(lib.tpi_star_reduce(P_all, N, m.hidden, src.data_ptr(), h_attn.data_ptr(), stream))
                check(lib.tpi_shards_layer_decode(cfg_p, 1, w, None, pos, B.TPI_PHASE_FFN, h_attn.data_ptr(),
                                                  P_one, WS_one, stream))
                check(lib.tpi_star_reduce(P_all, N, m.hidden, h_attn.data_ptr(), dst.data_ptr(), stream))
                win.release(l)
                win.prefetch(nxt[0] % Lf)
                nxt[0] += 1
                src, dst = dst, (h_b if dst is h_a else h_a)
            return src

        token(pos0)
        torch.cuda.current_stream().synchronize()      # not the copy stream: see window_leg
        r0 = win.read_ms()
        t = time.perf_counter()
        steps = max(1, min(2, args.window_steps))
        for i in range(steps):
            out = token(pos0 + 1 + i)
        torch.cuda.current_stream().synchronize()
        ms = (time.perf_counter() - t) * 1e3 / steps
        read_ms = (win.read_ms() - r0) / steps
        finite = bool(torch.isfinite(out).all().item())
        win.destroy()
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    gb = Lf * nbytes / 1e9
    return {
        "layers_per_token": Lf, "window_layers": Wn, "staging_buffers": 2, "reader_threads": args.window_file_readers,
        "files": D, "ms_per_token": round(ms, 2),
        "gb_per_token": round(gb, 3), "loader_gbps": round(gb / (ms * 1e-3), 2),
        "pread_ms_per_token": round(read_ms, 2), "pread_gbps": round(gb / (read_ms * 1e-3), 2) if read_ms > 0 else None,
        "link_peak_gbps_plain_copy": round(link_gbps, 2), "source": "files read through the page cache",
        "output_finite": finite,
    }


def window_blocks_variant(args, m, L, N, blobs, host, layout, cfg, KV_one, P_all, P_one, WS_one, h0, h_a, h_b, h_attn,
                          pos0, link_gbps, T):
    """The window at the paper's granularity: a window of w = --window-layers blocks, half of them attention
    blocks and half FFN blocks (w/2 slots each), and -- for T > 0 -- block retention (Prop. 6): the FFN
    block of every T-th layer is copied once and stays.  Decode is copy-bound here, so ms/token should
    follow the bytes that still have to cross the link.  The retained blocks' device home is shard 0's own
    region of the resident stack (identical bytes, no extra memory; the windowed run reads nothing else of it)."""
    import torch

    from paper_2410_00531_amd import binding as B
    from paper_2410_00531_amd import synth
    dev = h0.device
    w = args.window_layers - args.window_layers % 2
    n_a = layout["ffn_norm"][0]                                   # floats of the attention block
    n_f = layout["w_down"][0] + layout["w_down"][2] - n_a         # floats of the FFN block
    slots_a = torch.empty((w // 2) * n_a, dtype=torch.float32, device=dev)
    slots_f = torch.empty((w // 2) * n_f, dtype=torch.float32, device=dev)
    retained = {2 * l + 1 for l in range(L) if T > 0 and l % T == 0}
    blocks = []
    for l in range(L):
        blocks.append((host[l][:n_a], n_a * 4, 0, None))
        blocks.append((host[l][n_a:], n_f * 4, 1, blobs[l][0][n_a:] if (2 * l + 1) in retained else None))
    win = B.Window.from_blocks(blocks, [(slots_a, n_a * 4, w // 2), (slots_f, n_f * 4, w // 2)])
    win.calibrate()
    lib = B.lib()
    stream = torch.cuda.current_stream().cuda_stream
    cfg_p = C.byref(cfg)
    issued = [0]

    def prefetch_next():
        win.prefetch(issued[0] % (2 * L))
        issued[0] += 1

    for _ in range(w):
        prefetch_next()

    def check(rc):
        if rc != 0:
            raise RuntimeError(B.tpi_last_error())

    wv = (B.tpi_layer_weights * 1)()

    def token(pos):
        src, dst = h0, h_a
        for l in range(L):
            base = win.acquire(2 * l)
            for name in ("attn_norm", "w_qkv", "w_o"):
                setattr(wv[0], name, base + layout[name][0] * 4)
            check(lib.tpi_shards_layer_decode(cfg_p, 1, wv, KV_one[l], pos, B.TPI_PHASE_ATTN, src.data_ptr(),
                                              P_one, WS_one, stream))
            check(lib.tpi_star_reduce(P_all, N, m.hidden, src.data_ptr(), h_attn.data_ptr(), stream))
            win.release(2 * l)
            prefetch_next()
            base = win.acquire(2 * l + 1)
            for name in ("ffn_norm", "w_gate", "w_up", "w_down"):
                setattr(wv[0], name, base + (layout[name][0] - n_a) * 4)
            check(lib.tpi_shards_layer_decode(cfg_p, 1, wv, None, pos, B.TPI_PHASE_FFN, h_attn.data_ptr(),
                                              P_one, WS_one, stream))
            check(lib.tpi_star_reduce(P_all, N, m.hidden, h_attn.data_ptr(), dst.data_ptr(), stream))
            win.release(2 * l + 1)
            prefetch_next()
            src, dst = dst, (h_b if dst is h_a else h_a)
        return src

    token(pos0)                                  # warm-up token: brings the retained blocks in
    torch.cuda.current_stream().synchronize()      # not the copy stream: see window_leg
    bytes0 = win.bytes_copied()
    t = time.perf_counter()
    for i in range(args.window_steps):
        out = token(pos0 + 1 + i)
    torch.cuda.current_stream().synchronize()
    ms = (time.perf_counter() - t) * 1e3 / args.window_steps
    bytes1 = win.bytes_copied()
    finite = bool(torch.isfinite(out).all().item())
    win.destroy()
    per_token = (bytes1 - bytes0) / args.window_steps
    return {
        "window_blocks": w, "retain_every": T, "retained_ffn_blocks": len(retained),
        "retained_gb": round(len(retained) * n_f * 4 / 1e9, 2),
        "window_slots_gb": round((w // 2) * (n_a + n_f) * 4 / 1e9, 3),
        "ms_per_token": round(ms, 2), "h2d_gb_per_token": round(per_token / 1e9, 3),
        "pcie_gbps": round(per_token / (ms * 1e-3) / 1e9, 2),
        "copy_ms_per_token_at_link_peak": round(per_token / (link_gbps * 1e9) * 1e3, 2), "output_finite": finite,
    }


def window_prefill_leg(args, m, seed):
    """The favourable point of the sliding window: one shard's bf16 layer blobs stream from pinned host
    memory through --window-layers HBM slots while a LONG prompt is prefilled.  Per layer the shard then
    computes for longer than its blob takes to copy (the loose steady condition of the paper's Prop. 3
    holds), so the copies should disappear behind the compute; with batch-1 decode they cannot."""
    import torch

    from paper_2410_00531_amd import binding as B
    from paper_2410_00531_amd import synth
    dev = torch.device("cuda:0")
    n, L, Wn, D = args.window_prefill_tokens, args.window_prefill_layers, args.window_layers, 8
    Wn = min(Wn, L)
    h, d, sl, nq, nkv = m.hidden, m.head_dim, m.ffn_local, m.nq_local, m.nkv_local
    cfg = B.make_cfg(h, nq, nkv, d, sl, n, m.rms_eps, m.rope_base, dtype=B.TPI_BF16)
    layout, nbytes = synth.blob_layout_bytes(h, nq, nkv, d, sl, 2)
    gen = torch.Generator(device=dev); gen.manual_seed(seed + 9)
    dev_blobs, host = [], []
    for i in range(min(D, L)):                      # D distinct blobs; layer l uses blob l % D (same traffic)
        b = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        for name, (off, shape, item) in layout.items():
            cnt = 1
            for s_ in shape:
                cnt *= s_
            if item == 4:
                b[off:off + cnt * 4].view(torch.float32).normal_(1.0, 0.02, generator=gen)
            else:
                b[off:off + cnt * 2].view(torch.bfloat16).normal_(0.0, 0.02, generator=gen)
        hb = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        hb.copy_(b)
        dev_blobs.append(b); host.append(hb)
    D = len(dev_blobs)
    slots = torch.empty(Wn * nbytes, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def link_peak():
        """Practical peak of the link: plain pinned copies of whole blobs, best of several rounds (measured
        right after earlier phases released their memory the first rounds have read about half)."""
        best = 0.0
        for _ in range(6):
            e0.record()
            for i in range(D):
                slots[:nbytes].copy_(host[i], non_blocking=True)
            e1.record(); torch.cuda.synchronize()
            best = max(best, D * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        return best

    def views(base):
        w = (B.tpi_layer_weights * 1)()
        for name, (off, _, _) in layout.items():
            setattr(w[0], name, base + off)
        return w

    res_w = [views(b.data_ptr()) for b in dev_blobs]
    slot_w = {slots.data_ptr() + i * nbytes: views(slots.data_ptr() + i * nbytes) for i in range(Wn)}
    x32 = torch.randn((n, h), generator=gen, device=dev)
    x16 = x32.to(torch.bfloat16)
    ha32 = torch.empty_like(x32); ha16 = torch.empty_like(x16)
    hb32 = torch.empty_like(x32); hb16 = torch.empty_like(x16)
    part = torch.empty((n, h), dtype=torch.float32, device=dev)
    others = torch.zeros((n, h), dtype=torch.float32, device=dev)     # the other ranks' partials (read only)
    N = m.n_shards
    P = (C.c_void_p * N)(part.data_ptr(), *[others.data_ptr()] * (N - 1))
    kc = torch.zeros((L, 2, nkv, n, d), dtype=torch.bfloat16, device=dev)
    KV = [B.make_kv(kc[l, 0], kc[l, 1]) for l in range(L)]
    ws = torch.empty(B.tpi_workspace_bytes(cfg, n) // 4, dtype=torch.float32, device=dev)
    lib = B.lib(); stream = torch.cuda.current_stream().cuda_stream; cfg_p = C.byref(cfg)

    def check(rc):
        if rc != 0:
            raise RuntimeError(B.tpi_last_error())

    def prompt(get_layer, release_layer):
        s32, s16 = x32, x16
        for l in range(L):
            w = get_layer(l)
            check(lib.tpi_shard_layer_prefill(cfg_p, w, C.byref(KV[l]), 0, n, B.TPI_PHASE_ATTN, s16.data_ptr(),
                                              part.data_ptr(), ws.data_ptr(), stream))
            check(lib.tpi_star_reduce_bf16(P, N, n * h, s32.data_ptr(), ha32.data_ptr(), ha16.data_ptr(), stream))
            check(lib.tpi_shard_layer_prefill(cfg_p, w, None, 0, n, B.TPI_PHASE_FFN, ha16.data_ptr(),
                                              part.data_ptr(), ws.data_ptr(), stream))
            check(lib.tpi_star_reduce_bf16(P, N, n * h, ha32.data_ptr(), hb32.data_ptr(), hb16.data_ptr(), stream))
            release_layer(l)
            s32, s16 = hb32, hb16
        return s32

    def timed(fn, reps):
        fn(); torch.cuda.current_stream().synchronize()      # the compute stream only, at both ends
        t = time.perf_counter()
        for _ in range(reps):
            out = fn()
        torch.cuda.current_stream().synchronize()
        return (time.perf_counter() - t) * 1e3 / reps, out

    ms_res, out_res = timed(lambda: prompt(lambda l: res_w[l % D], lambda l: None), 2)
    ref = out_res.clone()
    link_gbps = link_peak()
    win = B.Window([host[l % D] for l in range(L)], slots, Wn, nbytes)
    copy_streams_tried = win.calibrate()
    for l in range(Wn):
        win.prefetch(l)
    nxt = [Wn]

    def release_layer(l):
        win.release(l)
        win.prefetch(nxt[0] % L)                  # slides on into the next prompt's layers
        nxt[0] += 1

    ms_win, out_win = timed(lambda: prompt(lambda l: slot_w[win.acquire(l)], release_layer), 2)
    same = bool(torch.equal(out_win, ref))
    win_copy_ms, win_copy_bytes = win.copy_stats()
    win.destroy()
    copy_ms = L * nbytes / (link_gbps * 1e9) * 1e3
    return {
        "workload": f"{m.name}-windowed-prefill-{n}-tokens-one-shard", "dtype": "bf16 weights, fp32 partials",
        "layers": L, "window_layers": Wn, "layer_blob_mb": round(nbytes / 1e6, 2),
        "ms_per_prompt_windowed": round(ms_win, 2), "ms_per_prompt_resident": round(ms_res, 2),
        "copy_ms_per_prompt_at_link_peak": round(copy_ms, 2), "link_peak_gbps_plain_copy": round(link_gbps, 2),
        "compute_over_copy": round(ms_res / copy_ms, 3),
        "hidden_fraction": round(min(1.0, 1.0 - (ms_win - ms_res) / copy_ms), 4),
        "copy_stream_effective_gbps": round(win_copy_bytes / (win_copy_ms * 1e-3) / 1e9, 2) if win_copy_ms > 0 else None,
        "windowed_equals_resident_bitwise": same,
        "copy_streams_tried_by_calibrate": copy_streams_tried,
        "position_in_process": "last leg, after the decode, prefill and probe legs created their streams",
    }


def prefill_leg(args, m, L, N, seed):
    """The prefill workload (70B-shaped 8-way shard, 512 tokens by default): prompt of --prefill-tokens tokens through the whole stack, all N shards emulated,
    bf16 weights and activations, fp32 partials star-reduced per layer (the reduce also emits the bf16 copy
    that feeds the next phase)."""
    import torch

    from paper_2410_00531_amd import binding as B
    dev = torch.device("cuda:0")
    n = args.prefill_tokens
    h, d, sl, nq, nkv = m.hidden, m.head_dim, m.ffn_local, m.nq_local, m.nkv_local
    dq, dkv = nq * d, nkv * d
    cfg = B.make_cfg(h, nq, nkv, d, sl, n, m.rms_eps, m.rope_base, dtype=B.TPI_BF16)
    sizes = [("w_qkv", (dq + 2 * dkv) * h), ("w_o", h * dq), ("w_gate", sl * h), ("w_up", sl * h), ("w_down", h * sl)]
    blob_elems = sum(s for _, s in sizes)
    gen = torch.Generator(device=dev); gen.manual_seed(seed + 5)
    blobs, norms = [], []
    for l in range(L):
        b = torch.empty((N, blob_elems), dtype=torch.bfloat16, device=dev)
        b.normal_(0.0, 0.02, generator=gen)
        g = torch.empty((N, 2, h), dtype=torch.float32, device=dev).normal_(1.0, 0.02, generator=gen)
        blobs.append(b); norms.append(g)
    kc = torch.zeros((L, N, 2, nkv, n, d), dtype=torch.bfloat16, device=dev)
    x32 = torch.randn((n, h), generator=gen, device=dev)
    x16 = x32.to(torch.bfloat16)
    Wl, KVl = [], []
    for l in range(L):
        ws_, ks_ = [], []
        for r in range(N):
            w = B.tpi_layer_weights()
            off = blobs[l][r].data_ptr()
            for name, sz in sizes:
                setattr(w, name, off); off += sz * 2
            # the norm is replicated on every device (Sec. 3.1): all shards of a layer name the same gains
            w.attn_norm = norms[l][0, 0].data_ptr(); w.ffn_norm = norms[l][0, 1].data_ptr()
            ws_.append(w); ks_.append(B.make_kv(kc[l, r, 0], kc[l, r, 1]))
        Wl.append(ws_); KVl.append(ks_)
    ws = torch.empty(B.tpi_workspace_bytes(cfg, n) // 4, dtype=torch.float32, device=dev)
    parts = torch.empty((N, n, h), dtype=torch.float32, device=dev)
    P = (C.c_void_p * N)(*[parts[r].data_ptr() for r in range(N)])
    ha32 = torch.empty_like(x32); ha16 = torch.empty_like(x16)
    hb32 = torch.empty_like(x32); hb16 = torch.empty_like(x16)
    lib = B.lib(); stream = torch.cuda.current_stream().cuda_stream; cfg_p = C.byref(cfg)

    def check(rc):
        if rc != 0:
            raise RuntimeError(B.tpi_last_error())

    def step(L=L):
        s32, s16 = x32, x16
        for l in range(L):
            for r in range(N):
                check(lib.tpi_shard_layer_prefill(cfg_p, C.byref(Wl[l][r]), C.byref(KVl[l][r]), 0, n,
                                                  B.TPI_PHASE_ATTN, s16.data_ptr(), parts[r].data_ptr(),
                                                  ws.data_ptr(), stream))
            check(lib.tpi_star_reduce_bf16(P, N, n * h, s32.data_ptr(), ha32.data_ptr(), ha16.data_ptr(), stream))
            for r in range(N):
                check(lib.tpi_shard_layer_prefill(cfg_p, C.byref(Wl[l][r]), None, 0, n, B.TPI_PHASE_FFN,
                                                  ha16.data_ptr(), parts[r].data_ptr(), ws.data_ptr(), stream))
            check(lib.tpi_star_reduce_bf16(P, N, n * h, ha32.data_ptr(), hb32.data_ptr(), hb16.data_ptr(), stream))
            s32, s16 = hb32, hb16
        return s32

    step(); torch.cuda.synchronize()
    K = args.prefill_steps
    t = time.perf_counter()
    for _ in range(K):
        out = step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t) * 1e3 / K

    # The N emulated shards are independent between the reduces: dealt to S streams (default priority), a
    # shard's small kernels (norm, rotary scatter, attention) run beside another shard's GEMMs.
    def step_streams(streams, wss, ev_in, ev_out):
        main = torch.cuda.current_stream()
        S = len(streams)
        s32, s16 = x32, x16

        def phase(l, ph, src16):
            ev_in.record(main)
            for st in streams:
                st.wait_event(ev_in)
            for r in range(N):
                check(lib.tpi_shard_layer_prefill(cfg_p, C.byref(Wl[l][r]), C.byref(KVl[l][r]) if ph == B.TPI_PHASE_ATTN else None,
                                                  0, n, ph, src16.data_ptr(), parts[r].data_ptr(),
                                                  wss[r % S].data_ptr(), streams[r % S].cuda_stream))
            for i, st in enumerate(streams):
                ev_out[i].record(st)
                main.wait_event(ev_out[i])

        for l in range(L):
            phase(l, B.TPI_PHASE_ATTN, s16)
            check(lib.tpi_star_reduce_bf16(P, N, n * h, s32.data_ptr(), ha32.data_ptr(), ha16.data_ptr(), stream))
            phase(l, B.TPI_PHASE_FFN, ha16)
            check(lib.tpi_star_reduce_bf16(P, N, n * h, ha32.data_ptr(), hb32.data_ptr(), hb16.data_ptr(), stream))
            s32, s16 = hb32, hb16
        return s32

    # All N shards of a phase in one set of launches (every kernel takes the shard from a grid dimension).
    wss_b = [torch.empty_like(ws) for _ in range(N)]
    WSb = (C.c_void_p * N)(*[t.data_ptr() for t in wss_b])
    Wb = [(B.tpi_layer_weights * N)(*Wl[l]) for l in range(L)]
    KVb = [(B.tpi_kv_layer * N)(*KVl[l]) for l in range(L)]

    def step_batched(L=L):
        s32, s16 = x32, x16
        for l in range(L):
            check(lib.tpi_shards_layer_prefill(cfg_p, N, Wb[l], KVb[l], 0, n, B.TPI_PHASE_ATTN, s16.data_ptr(), P, WSb, stream))
            check(lib.tpi_star_reduce_bf16(P, N, n * h, s32.data_ptr(), ha32.data_ptr(), ha16.data_ptr(), stream))
            check(lib.tpi_shards_layer_prefill(cfg_p, N, Wb[l], None, 0, n, B.TPI_PHASE_FFN, ha16.data_ptr(), P, WSb, stream))
            check(lib.tpi_star_reduce_bf16(P, N, n * h, ha32.data_ptr(), hb32.data_ptr(), hb16.data_ptr(), stream))
            s32, s16 = hb32, hb16
        return s32

    batched = None
    if not args.no_prefill_batched:
        def rel_diff(a, b):
            den = float(b.abs().max().item())
            return float((a - b).abs().max().item()) / (den if den > 0 else 1.0)

        ref1 = step(1).clone()                      # one layer both ways: the plans differ, the sums agree
        err_1 = rel_diff(step_batched(1), ref1)
        ref = step().clone()
        got = step_batched(); torch.cuda.synchronize()
        err_b = rel_diff(got, ref)                  # after L free-running layers rounding differences have grown
        t = time.perf_counter()
        for _ in range(K):
            step_batched()
        torch.cuda.synchronize()
        ms_b = (time.perf_counter() - t) * 1e3 / K
        B.tpi_prof_enable(B.TPI_STAGE_PREFILL_GEMM, 4 * L)
        step_batched(); torch.cuda.synchronize()
        gemm_ms_b, gemm_n_b = B.tpi_prof_read()
        B.tpi_prof_enable(B.TPI_STAGE_NONE, 0)
        batched = {"ms_per_prompt": round(ms_b, 3), "max_rel_diff_to_per_shard_calls_one_layer": float(f"{err_1:.3g}"),
                   "max_rel_diff_to_per_shard_calls_whole_stack": float(f"{err_b:.3g}"),
                   "gemm_launches": gemm_n_b, "gemm_total_ms": round(gemm_ms_b, 3)}
    del wss_b

    by_streams = {}
    for S in ([] if args.prefill_streams <= 1 else [args.prefill_streams]):
        streams = [torch.cuda.Stream() for _ in range(S)]
        wss = [torch.empty_like(ws) for _ in range(S)]
        ev_in = torch.cuda.Event(); ev_out = [torch.cuda.Event() for _ in range(S)]
        B.tpi_set_prefill_concurrency(S)            # the GEMM plans size their grids for 1/S of the chip
        ref = step().clone()                        # same plans on one stream: the results must be the same bits
        got = step_streams(streams, wss, ev_in, ev_out); torch.cuda.synchronize()
        same = bool(torch.equal(got, ref))
        t = time.perf_counter()
        for _ in range(K):
            step_streams(streams, wss, ev_in, ev_out)
        torch.cuda.synchronize()
        by_streams[S] = {"ms_per_prompt": round((time.perf_counter() - t) * 1e3 / K, 3), "output_equal_to_one_stream": same}
        B.tpi_set_prefill_concurrency(1)
        del streams, wss
    B.tpi_prof_enable(B.TPI_STAGE_PREFILL_GEMM, 4 * N * L)
    step(); torch.cuda.synchronize()
    gemm_ms, gemm_n = B.tpi_prof_read()
    B.tpi_prof_enable(B.TPI_STAGE_NONE, 0)
    gemm_flops = 2.0 * n * (h * (dq + 2 * dkv) + dq * h + 3 * h * sl)
    attn_flops = 2.0 * nq * d * n * (n + 1)
    total = (gemm_flops + attn_flops) * N * L
    peak = 2500.0
    ms_one_stream, arrangement = ms, "one shard per call, one stream"
    for S, v in by_streams.items():          # the prompt's time is the best arrangement of the same work
        if v["output_equal_to_one_stream"] and v["ms_per_prompt"] < ms:
            ms, arrangement = v["ms_per_prompt"], f"one shard per call, shards dealt to {S} streams"
    # sanity bound between two GPU arrangements of one layer (other GEMM plans, another attention kernel): half the
    # bf16 tolerance that each of them meets against the oracle in the parity tests
    if batched and batched["max_rel_diff_to_per_shard_calls_one_layer"] <= 1e-2 and batched["ms_per_prompt"] < ms:
        ms, arrangement = batched["ms_per_prompt"], f"all {N} shards per call (tpi_shards_layer_prefill)"
        gemm_ms, gemm_n = batched["gemm_total_ms"], batched["gemm_launches"]
    return {
        "workload": f"{m.name}-prefill-{n}-tokens", "dtype": "bf16 (fp32 accumulate, fp32 partials)",
        "layers": L, "shards_emulated": N, "steps": K, "ms_per_prompt": round(ms, 3),
        "arrangement": arrangement, "ms_per_prompt_one_stream": round(ms_one_stream, 3),
        "all_shards_per_call": batched,
        "prompt_tokens_per_s": round(n / (ms * 1e-3), 1), "tflop_per_prompt": round(total / 1e12, 2),
        "tflops": round(total / (ms * 1e-3) / 1e12, 1), "mfma_frac_of_peak_whole_step": round(total / (ms * 1e-3) / 1e12 / peak, 4),
        "gemm_kernels": {"launches": gemm_n, "total_ms": round(gemm_ms, 3),
                         "tflops": round(gemm_flops * N * L / (gemm_ms * 1e-3) / 1e12, 1) if gemm_n else None,
                         "frac_of_bf16_peak": round(gemm_flops * N * L / (gemm_ms * 1e-3) / 1e12 / peak, 4) if gemm_n else None,
                         "peak_tflops": peak},
        "reduce_gb_per_prompt": round(2 * L * (N + 2) * n * h * 4 / 1e9 + 2 * L * n * h * 2 / 1e9, 2),
        "shards_on_streams": {str(k): v for k, v in by_streams.items()} or None,
        "output_finite": bool(torch.isfinite(out).all().item()),
    }


# HBM bytes of one k_gate_up launch as the byte counters saw them (rocprofv3 --pmc FETCH_SIZE, then
# WRITE_SIZE, KiB per dispatch, each scaled by what the same counter reads for a plain 1 GiB device copy: FETCH_SIZE
# reads half of the copy's bytes (factor 2.0), WRITE_SIZE all of them (factor 1.0)).  A figure from separate profiler
# runs of this command, kept in profiles/; None for a workload those runs did not cover.
# "kernel_as_of": the commit whose k_gate_up the counters were read from; a later change to that kernel (stage_gate_up,
# RowStreamer) makes the figure stale until the two counter runs are repeated.
MEASURED_GATE_UP_TRAFFIC = {
    ("llama2-70b-shaped-tp8", 8): {"bytes": 1882007848,   # (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0) KiB x 1024 from the unrounded averages of that profile
                                   "source": "profiles/decode_70b_tp8_eight_shards_per_launch.md",
                                   "kernel_as_of": "6f5c362"},
}


def measured_traffic(m, n_launch_shards):
    hit = MEASURED_GATE_UP_TRAFFIC.get((m.name, n_launch_shards))
    return hit["bytes"] if hit else None


def measured_traffic_source(m, n_launch_shards):
    hit = MEASURED_GATE_UP_TRAFFIC.get((m.name, n_launch_shards))
    return {"profile": hit["source"], "kernel_as_of_commit": hit["kernel_as_of"]} if hit else None


def handover_probe_leg():
    """What chaining two dependent streaming stages costs on this chip (tpi_probe_handover): 4 GiB streamed in
    segments the size of a decode stage's weights, handed over inside the workgroup, across the chip inside one
    kernel, or by a kernel boundary.  us per hand-over = (time - time without hand-overs) / hand-overs."""
    from paper_2410_00531_amd import binding as B
    total = 4 << 30
    base = B.tpi_probe_handover(total, 2048, 0)
    out = {"bytes": total, "streaming_tb_per_s": round(base["tb_per_s"], 3), "streaming_us": round(base["us_total"], 1),
           "segments": {}}
    names = {1: "inside_the_workgroup", 2: "across_the_chip_in_one_kernel", 3: "kernel_boundary"}
    for kib in (16, 32, 64, 128):
        row = {}
        for mode in (1, 2, 3):
            r = B.tpi_probe_handover(total, kib, mode)
            n = r["segments"]
            d = {"us_per_hand_over": round((r["us_total"] - base["us_total"]) / max(n - 1, 1), 2),
                 "tb_per_s": round(r["tb_per_s"], 3), "results_ok": bool(r["results_ok"])}
            if mode == 2:
                d["first_to_last_workgroup_us"] = round(r["spread_us"], 2)
                d["last_result_to_next_use_us"] = round(r["chain_us"], 2)
            row[names[mode]] = d
        out["segments"][f"{r['segment_mb']:.1f} MB"] = row
    return out


def gemm_loop_probe_leg():
    """What paces the K loop of the prefill's 256x256 GEMM tile (tpi_probe_gemm_loop): the 8-shard down projection of
    the 70B shape as the library runs it, and with the loads into LDS, the fragment reads from LDS or the matrix
    instructions taken out of the kernel, one or two at a time (those variants compute nothing meaningful)."""
    from paper_2410_00531_amd import binding as B
    names = {0: "complete_loop", 1: "without_loads", 2: "without_fragment_reads", 4: "without_matrix_instructions",
             3: "matrix_instructions_only", 5: "fragment_reads_only", 6: "loads_only"}
    full = B.tpi_probe_gemm_loop(0, reps=10)
    out = {"workload": "8 shards x [512 x 3584] . [8192 x 3584]^T, bf16, 256x256 tiles",
           "tflop_per_launch": round(full["tflop_per_launch"], 4), "result_ok": bool(full["result_ok"] == 1),
           "us_per_launch": {}}
    for leave_out in (0, 1, 2, 4, 3, 5, 6):
        r = full if leave_out == 0 else B.tpi_probe_gemm_loop(leave_out, reps=10)
        out["us_per_launch"][names[leave_out]] = round(r["us_per_launch"], 1)
    out["tflops_complete_loop"] = round(full["tflops"], 1)
    out["tflops_matrix_instructions_only"] = round(full["tflop_per_launch"] / (out["us_per_launch"]["matrix_instructions_only"] * 1e-6), 1)
    return out


def config2_leg(args):
    """BASELINE's other configuration (8B-shaped, 4 shards x 32 layers, KV length 512), a short decode leg of its own:
    this script again as a child process, once the big stack has been released; its JSON line is returned in brief."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--workload", "llama3.1-8b-shaped-tp4", "--steps", str(args.steps),
           "--warmup", str(args.warmup), "--no-window", "--no-prefill", "--no-token-ends", "--no-cpu-baseline", "--no-config2"]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    if res.returncode != 0:
        return {"error": (res.stderr or res.stdout)[-400:]}
    r = json.loads(res.stdout.strip().splitlines()[-1])
    one = r.get("one_shard") or {}
    return {"workload": r["config"]["workload"], "layers": r["config"]["layers"], "shards_emulated": r["config"]["shards_emulated"],
            "kv_len": r["config"]["kv_len"], "weights_gb": r["config"]["weights_gb"], "steps": r["steps"],
            "ms_per_token": r["value"], "algorithmic_gb_per_token": r["algorithmic_gb_per_token"],
            "hbm_gbps": r["hbm_gbps"], "hbm_frac_of_peak": r["hbm_frac_of_peak"],
            "star_reduce_arrangements": r.get("star_reduce_arrangements"),
            "one_shard": {k: one.get(k) for k in ("ms_per_token", "hbm_frac_of_peak", "ms_per_token_reduce_folded_into_phase",
                                                  "hbm_frac_of_peak_reduce_folded")},
            "gate_up_kernel": {k: r["roofline"][k] for k in ("achieved", "frac", "avg_launch_us", "bytes_per_launch")},
            "output_finite": r["output_finite"]}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the N shards of the tensor-parallel layer are emulated "
              "on it and no multi-GPU figure exists. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2410_00531_amd import binding as B
    from paper_2410_00531_amd import configs, synth

    m = configs.BY_NAME[args.workload]
    L = args.layers or m.n_layers
    N = m.n_shards
    kv_len = args.kv_len or {"llama2-70b-shaped-tp8": 1024, "llama3.1-8b-shaped-tp4": 512, "tiny": 16}[args.workload]
    K, W = args.steps, args.warmup
    n_tokens_total = 9 * (K + W) + 8
    max_seq = kv_len + n_tokens_total
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B.lib()
    cfg = B.make_cfg(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, max_seq, m.rms_eps, m.rope_base)
    layout, blob_floats = blob_layout(m)
    assert blob_floats == m.layer_shard_params()

    # ---- synthetic stack, drawn on the device (seeded) ------------------------------------------
    gen = torch.Generator(device=dev); gen.manual_seed(args.seed)
    t0 = time.time()
    blobs = []                                            # [layer] tensor [N][blob_floats]
    for l in range(L):
        b = torch.empty((N, blob_floats), dtype=torch.float32, device=dev)
        b.normal_(0.0, synth.WEIGHT_STD, generator=gen)
        for name in ("attn_norm", "ffn_norm"):
            off, _, n = layout[name]
            b[:, off:off + n] += 1.0
        blobs.append(b)
    kc = torch.zeros((L, N, 2, m.nkv_local, max_seq, m.head_dim), dtype=torch.float32, device=dev)
    kc[:, :, :, :, :kv_len].normal_(0.0, 1.0, generator=gen)
    h0 = torch.randn(m.hidden, generator=gen, device=dev)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    # ---- pre-marshalled argument blocks ---------------------------------------------------------
    esz = 4
    W_all, KV_all, W_one, KV_one = [], [], [], []
    for l in range(L):
        wl = (B.tpi_layer_weights * N)()
        kl = (B.tpi_kv_layer * N)()
        for r in range(N):
            base = blobs[l][r].data_ptr()
            for name in synth.TENSOR_ORDER:
                setattr(wl[r], name, base + layout[name][0] * esz)
            kl[r].k = kc[l, r, 0].data_ptr(); kl[r].v = kc[l, r, 1].data_ptr()
        W_all.append(wl); KV_all.append(kl)
        W_one.append((B.tpi_layer_weights * 1)(wl[0])); KV_one.append((B.tpi_kv_layer * 1)(kl[0]))
    ws_bytes = B.tpi_workspace_bytes(cfg, 1)
    ws = torch.empty((N, ws_bytes // 4), dtype=torch.float32, device=dev)
    partials = torch.zeros((N, m.hidden), dtype=torch.float32, device=dev)
    P_all = (C.c_void_p * N)(*[partials[r].data_ptr() for r in range(N)])
    WS_all = (C.c_void_p * N)(*[ws[r].data_ptr() for r in range(N)])
    P_one = (C.c_void_p * 1)(partials[0].data_ptr())
    WS_one = (C.c_void_p * 1)(ws[0].data_ptr())
    h_a = torch.empty_like(h0); h_b = torch.empty_like(h0); h_attn = torch.empty_like(h0)

    lib = B.lib()
    stream = torch.cuda.current_stream().cuda_stream
    cfg_p = C.byref(cfg)

    def check(rc):
        if rc != 0:
            raise RuntimeError(B.tpi_last_error())

    last_out = [h0]
    fold_all = not args.separate_reduce

    def token(pos, all_shards=True, fused=None):
        """One token through the stack; returns the output hidden state tensor.  All shards: batched
        phase launches + star reduce kernels.  One shard: one device's view; the 8-way reduce runs over
        its own partial and the 7 peers' partial buffers, either as the separate star-reduce launch or
        (fused) folded into the phase's last stage."""
        src, dst = h0, h_a
        if all_shards and (fold_all if fused is None else fused):
            # every phase with its star reduce folded into the row-parallel stage: 2 calls, 5 launches per layer
            for l in range(L):
                check(lib.tpi_shards_layer_decode_reduce(cfg_p, N, W_all[l], KV_all[l], pos, B.TPI_PHASE_ATTN, src.data_ptr(),
                                                         h_attn.data_ptr(), WS_all, stream))
                check(lib.tpi_shards_layer_decode_reduce(cfg_p, N, W_all[l], None, pos, B.TPI_PHASE_FFN, h_attn.data_ptr(),
                                                         dst.data_ptr(), WS_all, stream))
                src, dst = dst, (h_b if dst is h_a else h_a)
        elif all_shards:
            for l in range(L):
                check(lib.tpi_shards_layer_decode(cfg_p, N, W_all[l], KV_all[l], pos, B.TPI_PHASE_ATTN, src.data_ptr(),
                                                  P_all, WS_all, stream))
                check(lib.tpi_star_reduce(P_all, N, m.hidden, src.data_ptr(), h_attn.data_ptr(), stream))
                check(lib.tpi_shards_layer_decode(cfg_p, N, W_all[l], None, pos, B.TPI_PHASE_FFN, h_attn.data_ptr(),
                                                  P_all, WS_all, stream))
                check(lib.tpi_star_reduce(P_all, N, m.hidden, h_attn.data_ptr(), dst.data_ptr(), stream))
                src, dst = dst, (h_b if dst is h_a else h_a)
        elif not fused:
            for l in range(L):
                check(lib.tpi_shards_layer_decode(cfg_p, 1, W_one[l], KV_one[l], pos, B.TPI_PHASE_ATTN, src.data_ptr(),
                                                  P_one, WS_one, stream))
                check(lib.tpi_star_reduce(P_all, N, m.hidden, src.data_ptr(), h_attn.data_ptr(), stream))
                check(lib.tpi_shards_layer_decode(cfg_p, 1, W_one[l], None, pos, B.TPI_PHASE_FFN, h_attn.data_ptr(),
                                                  P_one, WS_one, stream))
                check(lib.tpi_star_reduce(P_all, N, m.hidden, h_attn.data_ptr(), dst.data_ptr(), stream))
                src, dst = dst, (h_b if dst is h_a else h_a)
        else:
            ws0 = ws[0].data_ptr()
            for l in range(L):
                check(lib.tpi_shard_layer_decode_reduce(cfg_p, W_one[l], KV_one[l], pos, B.TPI_PHASE_ATTN, src.data_ptr(),
                                                        N, 0, P_all, h_attn.data_ptr(), ws0, stream))
                check(lib.tpi_shard_layer_decode_reduce(cfg_p, W_one[l], None, pos, B.TPI_PHASE_FFN, h_attn.data_ptr(),
                                                        N, 0, P_all, dst.data_ptr(), ws0, stream))
                src, dst = dst, (h_b if dst is h_a else h_a)
        last_out[0] = src
        return src

    def timed(n_steps, pos0, all_shards):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_steps)]
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(n_steps):
            ev[i][0].record()
            token(pos0 + i, all_shards)
            ev[i][1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t
        per = sorted(a.elapsed_time(b) for a, b in ev)
        return wall * 1e3 / n_steps, per[len(per) // 2], per[0]

    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    def leg(all_shards):
        """W warm-up tokens, K timed tokens, then the same K tokens again with HIP events
        around every launch of the dominant kernel (gate/up)."""
        nonlocal pos
        for i in range(W):
            token(pos + i, all_shards)
        pos += W
        ms, med, mn = timed(K, pos, all_shards); pos += K
        B.tpi_prof_enable(B.TPI_STAGE_GATE_UP, K * L)
        timed(K, pos, all_shards); pos += K
        k_ms, k_n = B.tpi_prof_read()
        B.tpi_prof_enable(B.TPI_STAGE_NONE, 0)
        return ms, med, k_ms, k_n

    pos = kv_len
    ms_all = med_all = gu_ms = ms_one = med_one = gu1_ms = float("nan")
    gu_n = gu1_n = 0
    if args.mode in ("both", "all"):
        ms_all, med_all, gu_ms, gu_n = leg(True)
    reduce_cmp = None
    if args.mode in ("both", "all") and fold_all:
        # the same step with the star reduces as launches of their own (the partial vectors go through memory):
        # same bits, 7 launches per layer instead of 5
        out_f = token(pos, True, True).clone()
        out_s = token(pos, True, False).clone()      # same position: rewrites the same cache slot with the same values
        pos += 1
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(K):
            token(pos + i, True, False)
        torch.cuda.synchronize()
        reduce_cmp = {"ms_per_token_separate_reduce_launches": round((time.perf_counter() - t) * 1e3 / K, 4),
                      "folded_equals_separate_bitwise": bool(torch.equal(out_f, out_s))}
        pos += K
    token(pos, True, False); pos += 1              # fills the peer partial buffers the one-shard legs read
    if args.mode in ("both", "one"):
        # one device's shard (peer partials stay as the last full step left them)
        ms_one, med_one, gu1_ms, gu1_n = leg(False)
    if args.mode == "one":
        ms_all, med_all, gu_ms, gu_n = ms_one, med_one, gu1_ms, gu1_n

    fused_ms = None
    if args.mode in ("both", "one") and not args.no_fused:
        for i in range(W):
            token(pos + i, False, True)
        pos += W
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(K):
            token(pos + i, False, True)
        torch.cuda.synchronize()
        fused_ms = (time.perf_counter() - t) * 1e3 / K
        pos += K

    assert pos <= max_seq
    torch.cuda.synchronize()
    finite = bool(torch.isfinite(last_out[0]).all().item())

    mid_pos = kv_len + W + K // 2
    bytes_all = token_bytes(m, N, N, L, mid_pos)
    bytes_one = token_bytes(m, 1, N, L, mid_pos)
    gbps_all = bytes_all / (ms_all * 1e-3) / 1e9
    gbps_one = bytes_one / (ms_one * 1e-3) / 1e9 if args.mode != "all" else float("nan")
    n_launch_shards = 1 if args.mode == "one" else N
    if args.mode == "one":
        bytes_all, gbps_all = bytes_one, gbps_one
    gu_bytes = stage_bytes(m, n_launch_shards, mid_pos)["gate_up"]
    gu_avg_ms = gu_ms / max(gu_n, 1)
    gu_gbps = gu_bytes / (gu_avg_ms * 1e-3) / 1e9 if gu_n else 0.0
    gu1_bytes = stage_bytes(m, 1, mid_pos)["gate_up"]
    gu1_avg_ms = gu1_ms / max(gu1_n, 1)

    result = {
        "metric": "decode_ms_per_token",
        "value": round(ms_all, 4),
        "unit": "ms/token",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_all, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{m.name}-resident-decode" + ("-one-shard" if args.mode == "one" else ""),
                   "layers": L, "shards_emulated": n_launch_shards, "shards_reduced": N,
                   "hidden": m.hidden, "q_heads_per_shard": m.nq_local, "kv_heads_per_shard": m.nkv_local,
                   "head_dim": m.head_dim, "ffn_per_shard": m.ffn_local, "kv_len": kv_len, "batch": 1,
                   "weights_gb": round(L * N * blob_floats * 4 / 1e9, 2)},
        "tokens_per_s": round(1e3 / ms_all, 3),
        "ms_per_token_median_events": round(med_all, 4),
        "algorithmic_gb_per_token": round(bytes_all / 1e9, 3),
        "hbm_gbps": round(gbps_all, 1),
        "hbm_frac_of_peak": round(gbps_all / HBM_PEAK_GBPS, 4),
        # the timed step calls tpi_shards_layer_decode_reduce (star reduce folded into the row-parallel stage)
        # unless --separate-reduce; the other arrangement and the bitwise comparison of the two:
        "star_reduce": ("separate launches" if not fold_all else "folded into the row-parallel stage") if args.mode != "one" else None,
        "star_reduce_arrangements": reduce_cmp,
        "one_shard": None if args.mode == "all" else {"ms_per_token": round(ms_one, 4), "ms_per_token_median_events": round(med_one, 4),
                      "tokens_per_s": round(1e3 / ms_one, 2),
                      "algorithmic_gb_per_token": round(bytes_one / 1e9, 3), "hbm_gbps": round(gbps_one, 1),
                      "hbm_frac_of_peak": round(gbps_one / HBM_PEAK_GBPS, 4),
                      "gate_up_kernel_avg_us": round(gu1_avg_ms * 1e3, 2),
                      "gate_up_kernel_gbps": round(gu1_bytes / (gu1_avg_ms * 1e-3) / 1e9, 1) if gu1_n else None,
                      # the same pass through the entry point that sums the peers' partials in the epilogue of the
                      # row-parallel kernels (5 launches per layer instead of 7): what a device of the star would call
                      "ms_per_token_reduce_folded_into_phase": round(fused_ms, 4) if fused_ms else None,
                      "hbm_gbps_reduce_folded": round(bytes_one / (fused_ms * 1e-3) / 1e9, 1) if fused_ms else None,
                      "hbm_frac_of_peak_reduce_folded": round(bytes_one / (fused_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4) if fused_ms else None},
        "roofline": {"kernel": f"k_gate_up (RMSNorm + gate/up GEMV + SiLU gate, {n_launch_shards} shard(s) per launch)",
                     "bound": "hbm", "achieved": round(gu_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gu_gbps / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(m, n_launch_shards),
                     "traffic_source": measured_traffic_source(m, n_launch_shards),
                     "bytes_per_launch": gu_bytes, "avg_launch_us": round(gu_avg_ms * 1e3, 2), "launches": gu_n},
        "output_finite": finite,
        "setup_s": round(setup_s, 1),
    }
    # ---- the master's work outside the layers --------------------------------------------------------
    if not args.no_token_ends:
        result["token_ends"] = token_ends_leg(args, m, result["value"])

    # ---- one shard with its weights streamed through a sliding window (pinned host -> HBM) --------
    if not args.no_window and args.mode in ("both", "one"):
        result["window"] = window_leg(args, m, L, N, blobs, layout, blob_floats, cfg, KV_one, P_all, P_one, WS_one,
                                      h0, h_a, h_b, h_attn, kv_len + n_tokens_total - args.window_steps - 2,
                                      ms_one)

    # ---- CPU baseline: the oracle as it stands, on a bounded sample ------------------------------
    if not args.no_cpu_baseline:
        from oracle import tpi_oracle as O
        oc = O.ShardCfg(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, max_seq, m.rms_eps, m.rope_base)
        w = {name: blobs[0][0][layout[name][0]:layout[name][0] + layout[name][2]].reshape(layout[name][1]).cpu().numpy()
             for name in synth.TENSOR_ORDER}
        Kc = kc[0, 0, 0].cpu().numpy().copy(); Vc = kc[0, 0, 1].cpu().numpy().copy()
        x = h0.cpu().numpy()
        reps, spent = 0, 0.0
        while spent < args.cpu_seconds and reps < 100000:
            t = time.perf_counter()
            pa = O.attn_block(oc, w["attn_norm"], w["w_qkv"], w["w_o"], Kc, Vc, kv_len, x)
            O.ffn_block(oc, w["ffn_norm"], w["w_gate"], w["w_up"], w["w_down"], pa.astype(np.float32))
            O.reduce_seq_f32([pa.astype(np.float32)] * N, x)
            spent += time.perf_counter() - t
            reps += 1
        per_layer_shard_ms = spent / reps * 1e3
        result["cpu_baseline"] = {
            "value": round(per_layer_shard_ms * L * N, 1), "unit": "ms/token", "cores": O.num_threads(),
            "kind": "oracle",
            "sample": f"{reps} x one layer of one shard (attention block + FFN block + one {N}-way reduce) at the "
                      f"workload's shape, {per_layer_shard_ms:.2f} ms each, scaled x{L} layers x{N} shards",
            "host_cores_seen": os.cpu_count(),
        }
        # the same sample on ONE thread
        n_thr = O.num_threads()
        O.set_num_threads(1)
        reps1, spent1 = 0, 0.0
        while spent1 < args.cpu_seconds / 2 and reps1 < 100000:
            t = time.perf_counter()
            pa = O.attn_block(oc, w["attn_norm"], w["w_qkv"], w["w_o"], Kc, Vc, kv_len, x)
            O.ffn_block(oc, w["ffn_norm"], w["w_gate"], w["w_up"], w["w_down"], pa.astype(np.float32))
            O.reduce_seq_f32([pa.astype(np.float32)] * N, x)
            spent1 += time.perf_counter() - t
            reps1 += 1
        O.set_num_threads(n_thr)
        result["cpu_baseline"]["single_thread"] = {
            "value": round(spent1 / reps1 * 1e3 * L * N, 1), "unit": "ms/token", "cores": 1,
            "sample": f"{reps1} x the same layer-shard, {spent1 / reps1 * 1e3:.2f} ms each, scaled x{L} layers x{N} shards"}
        # the prefill on the oracle: one layer of one shard at the prompt length of the prefill leg (bf16-valued inputs
        # widened, as in the parity tests), scaled to the whole stack and stated as scaled
        if not args.no_prefill and args.mode == "both":
            n_p = args.prefill_tokens
            wb = {k: (v if k.endswith("_norm") else synth.to_bf16_grid(v)) for k, v in w.items()}
            xp = synth.to_bf16_grid(np.random.default_rng(args.seed).standard_normal((n_p, m.hidden)).astype(np.float32))
            ocp = O.ShardCfg(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local, n_p, m.rms_eps, m.rope_base)
            Kp = np.zeros((m.nkv_local, n_p, m.head_dim), np.float32); Vp = np.zeros_like(Kp)
            t = time.perf_counter()
            pa = O.attn_block(ocp, wb["attn_norm"], wb["w_qkv"], wb["w_o"], Kp, Vp, 0, xp)
            O.ffn_block(ocp, wb["ffn_norm"], wb["w_gate"], wb["w_up"], wb["w_down"], xp)
            one_ms = (time.perf_counter() - t) * 1e3
            result["cpu_baseline"]["prefill"] = {
                "value": round(one_ms * L * N, 1), "unit": "ms/prompt", "cores": O.num_threads(), "kind": "oracle",
                "sample": f"1 x one layer of one shard, {n_p} prompt tokens (attention block + FFN block), {one_ms:.0f} ms, "
                          f"scaled x{L} layers x{N} shards (reduces not included)"}
    # ---- bf16 prefill of the same stack (the fp32 stack is released first: both do not fit) -------
    want_prefill = not args.no_prefill and args.mode == "both"
    if want_prefill:
        del blobs, kc, W_all, KV_all, W_one, KV_one
        torch.cuda.empty_cache()
        result["prefill"] = prefill_leg(args, m, L, N, args.seed)
        torch.cuda.empty_cache()
    # ---- the window where PCIe allows hiding: a long prompt through one shard's windowed layers ---
    # Runs late in the process on purpose, after many streams have been created: the window picks a copy stream that
    # does not share a hardware queue with the compute stream (tpi_window_calibrate).  Without that its copies
    # took turns with the kernels whenever the two streams met on one of the process's four hardware queues.
    if not args.no_window and not args.no_window_prefill and args.mode == "both":
        if "blobs" in dir():
            del blobs, kc, W_all, KV_all, W_one, KV_one
        torch.cuda.empty_cache()
        result.setdefault("window", {})["long_prompt_prefill"] = window_prefill_leg(args, m, args.seed)
        torch.cuda.empty_cache()
    # ---- what a hand-over between dependent stages costs (why one shard per launch stays latency-bound) ----
    if not args.no_handover_probe and args.mode == "both":
        if "blobs" in dir():
            del blobs, kc, W_all, KV_all, W_one, KV_one
        torch.cuda.empty_cache()
        result["handover_probe"] = handover_probe_leg()
    # ---- what paces the prefill's GEMM loop -------------------------------------------------------
    if not args.no_gemm_probe and not args.no_prefill and args.mode == "both":
        if "blobs" in dir():
            del blobs, kc, W_all, KV_all, W_one, KV_one
        torch.cuda.empty_cache()
        result["gemm_loop_probe"] = gemm_loop_probe_leg()
    # ---- the benchmark spec's other configuration, in brief ------------------------------------------
    if not args.no_config2 and args.mode == "both" and args.workload == "llama2-70b-shaped-tp8":
        if "blobs" in dir():
            del blobs, kc, W_all, KV_all, W_one, KV_one
        torch.cuda.empty_cache()
        result["config2"] = config2_leg(args)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
