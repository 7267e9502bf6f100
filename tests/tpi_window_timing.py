"""One case of the measured-window-times check (see tests/test_gpu_window.py), run as a process of its own:
python tests/tpi_window_timing.py <pad> <T>.  Exit status 0 and one line of figures when the windowed run took
the time the scheduler oracle predicts from the measured block and copy durations.

Why a process of its own: a process has four hardware queues, and the streams it has created share them.  Once
many streams exist (PyTorch's stream pool after any torch.cuda.Stream(), the streams of earlier windows), the
window's copy stream can land on the hardware queue that also carries the compute stream, and the marker that
follows a copy then holds back the kernels queued behind it: copies and compute take turns instead of
overlapping (windowed time = compute + copies).  In a fresh process the two streams have queues of their own."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for p in (ROOT, os.path.dirname(os.path.abspath(__file__))):
    if p not in sys.path:
        sys.path.insert(0, p)

from oracle import window_model as M                      # noqa: E402
from paper_2410_00531_amd import binding as B             # noqa: E402
from paper_2410_00531_amd import synth                    # noqa: E402

ATTN_TENSORS = ("attn_norm", "w_qkv", "w_o")
FFN_TENSORS = ("ffn_norm", "w_gate", "w_up", "w_down")


def _block_layout(shapes, names):
    off, out = 0, {}
    for name in names:
        n = int(np.prod(shapes[name]))
        out[name] = (off, n)
        off += n
    return out, off


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def run_case(pad, T, extra_streams=0, strict=True, calibrate=False):
    """Sec. 3.3 with numbers measured on this GPU: the block times t_attn, t_ffn and the copy times tau_attn,
    tau_ffn are measured with events, fed into the oracle's event simulation of the scheduler, and the
    windowed run must then take the time the simulation predicts and wait at the blocks where it predicts
    waits.  pad = 0 is batch-1 decode, where the copies take far longer than the blocks (Prop. 3 fails:
    every streamed block waits); with pad = 1 every block is followed by dense fp32 matrix products on the same
    stream (one after an attention block, three after an FFN block) -- a stand-in for a longer block
    computation, the scheduler sees only its duration -- and the loose steady condition holds: after the
    first window nothing waits.  T = 2 keeps the FFN block of every second layer resident (Prop. 6)."""
    # extra_streams: streams created (and used once) before the window exists -- they take shares of the process's
    # hardware queues, which decides whether the window's copy stream gets a queue of its own
    keep_streams = [torch.cuda.Stream() for _ in range(extra_streams)]
    for st in keep_streams:
        with torch.cuda.stream(st):
            torch.zeros(1, device="cuda")
    torch.cuda.synchronize()
    h, nq, nkv, d, sl = 2048, 16, 4, 128, 5632               # h = nq * d, so the paper's block formulas apply
    L, w, n_tokens, pos0, max_seq = 6, 4, 3, 5, 16
    cfg = B.make_cfg(h, nq, nkv, d, sl, max_seq)
    shapes = synth.shard_tensor_shapes(h, nq, nkv, d, sl)
    lay_a, n_a = _block_layout(shapes, ATTN_TENSORS)
    lay_f, n_f = _block_layout(shapes, FFN_TENSORS)
    # the slots of a window of w blocks are Prop. 5's peak for a worker (one shard holding all heads: p = 1)
    assert (w // 2) * (n_a + n_f) == M.peak_worker_params(w, h, nq, nkv, sl, 1.0)
    rng = np.random.default_rng(9)
    host = []
    for l in range(L):
        wts = synth.make_layer_shard(rng, h, nq, nkv, d, sl)
        for lay, n in ((lay_a, n_a), (lay_f, n_f)):
            blob = torch.empty(n, dtype=torch.float32).pin_memory()
            for name, (off, cnt) in lay.items():
                blob[off:off + cnt] = torch.from_numpy(wts[name].reshape(-1))
            host.append(blob)
    x = torch.from_numpy(rng.standard_normal(h).astype(np.float32)).cuda()
    part = torch.empty_like(x); h_attn = torch.empty_like(x); out = torch.empty_like(x)
    ws = torch.empty(B.tpi_workspace_bytes(cfg, 1) // 4, device="cuda")
    caches = [(torch.zeros((nkv, max_seq, d), device="cuda"), torch.zeros((nkv, max_seq, d), device="cuda")) for _ in range(L)]
    kv = [B.make_kv(K, V) for K, V in caches]

    def weights(attn_base, ffn_base):
        wv = B.tpi_layer_weights()
        for name, (off, _) in lay_a.items():
            setattr(wv, name, attn_base + off * 4)
        for name, (off, _) in lay_f.items():
            setattr(wv, name, ffn_base + off * 4)
        return wv

    filler = torch.randn((4096, 4096), device="cuda")
    sink = torch.empty_like(filler)

    def attn_block(l, base, pos):
        B.tpi_shard_layer_decode(cfg, weights(base, 0), kv[l], pos, B.TPI_PHASE_ATTN, x, part, ws)
        B.tpi_star_reduce([part], x, h_attn)
        for _ in range(pad):
            torch.mm(filler, filler, out=sink)

    def ffn_block(l, base, pos):
        B.tpi_shard_layer_decode(cfg, weights(0, base), None, pos, B.TPI_PHASE_FFN, h_attn, part, ws)
        B.tpi_star_reduce([part], h_attn, out)
        for _ in range(3 * pad):
            torch.mm(filler, filler, out=sink)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    # t_attn, t_ffn: resident blocks, medians over the layers of two tokens (the reduce belongs to the block here,
    # so t_all-reduce = 0 in the model)
    dev = [b.cuda() for b in host]
    t_a, t_f = [], []
    for t in range(3):
        for l in range(L):
            e0, e1, e2 = ev(), ev(), ev()
            e0.record(); attn_block(l, dev[2 * l].data_ptr(), pos0)
            e1.record(); ffn_block(l, dev[2 * l + 1].data_ptr(), pos0)
            e2.record(); torch.cuda.synchronize()
            if t:
                t_a.append(e0.elapsed_time(e1)); t_f.append(e1.elapsed_time(e2))
    t_attn, t_ffn = _median(t_a), _median(t_f)
    # tau_attn, tau_ffn: the window's own copies with nothing else running (no stream beside the window's is created)
    taus = []
    for b, n in ((0, n_a), (1, n_f)):
        dst = torch.empty(2 * n, device="cuda")
        probe = B.Window.from_blocks([(host[b], n * 4, 0, None)], [(dst, n * 4, 2)])
        ts = []
        for i in range(6):
            probe.prefetch(0); probe.acquire(0); probe.release(0)
            ms, _ = probe.copy_stats()
            ts.append(ms)
        probe.destroy()
        per = [ts[i] - ts[i - 1] for i in range(2, 6)]     # first_begin .. last_done grows by one copy per round
        taus.append(_median(per))
    tau_attn, tau_ffn = taus

    # the windowed run, with an event pair around every block's wait
    retained = {2 * l + 1 for l in range(L) if T > 0 and l % T == 0}
    homes = {b: torch.empty(n_f, device="cuda") for b in retained}
    slots_a = torch.empty((w // 2) * n_a, device="cuda"); slots_f = torch.empty((w // 2) * n_f, device="cuda")
    win = B.Window.from_blocks([(host[b], host[b].numel() * 4, b % 2, homes.get(b)) for b in range(2 * L)],
                               [(slots_a, n_a * 4, w // 2), (slots_f, n_f * 4, w // 2)])
    tried = win.calibrate() if calibrate else 0
    total = 2 * L * n_tokens
    issued = [0]

    def prefetch_next():
        if issued[0] < total:
            win.prefetch(issued[0] % (2 * L)); issued[0] += 1

    torch.cuda.synchronize()
    begin = ev(); begin.record()
    for _ in range(w):
        prefetch_next()
    marks = []
    for i in range(total):
        b, l = i % (2 * L), (i % (2 * L)) // 2
        before, after = ev(), ev()
        before.record()
        base = win.acquire(b)
        after.record()                                   # reached when the block's copy has landed
        (ffn_block if b % 2 else attn_block)(l, base, pos0 + i // (2 * L))
        win.release(b)
        prefetch_next()
        marks.append((before, after))
    end = ev(); end.record()
    torch.cuda.synchronize()
    win.destroy()
    measured = begin.elapsed_time(end)
    stalls = [a.elapsed_time(c) for a, c in marks]

    r = M.simulate(t_attn, t_ffn, 0.0, tau_attn, tau_ffn, n_layers=L, w=w, tokens=n_tokens, retain_T=T or None)
    # the window loads a retained block on first use, the model has it resident from the start: add those copies
    predicted = r.finish + (len(retained) * tau_ffn if tau_ffn > t_ffn else 0.0)
    info = (f"t_attn {t_attn:.3f} t_ffn {t_ffn:.3f} tau_attn {tau_attn:.3f} tau_ffn {tau_ffn:.3f} ms; "
            f"measured {measured:.2f} ms, predicted {predicted:.2f} ms" + (f", copy streams tried {tried}" if calibrate else ""))
    if not strict:
        return info
    assert abs(measured - predicted) <= 0.25 * predicted, info
    # where the model says a block waits for most of a copy, it does; where it says nothing waits, nothing does
    # (the last token: every retained block is in by then)
    nb = 2 * L
    long_wait, no_wait = 0.5 * min(tau_attn, tau_ffn), 0.15 * max(tau_attn, t_attn)
    for i in range(total - nb, total):
        if r.stalls[i] >= min(tau_attn, tau_ffn):
            assert stalls[i] >= long_wait, f"block {i}: model waits {r.stalls[i]:.3f} ms, run waited {stalls[i]:.3f}; " + info
        if r.stalls[i] == 0.0:
            assert stalls[i] <= no_wait, f"block {i}: model does not wait, run waited {stalls[i]:.3f} ms; " + info
    if pad:
        assert M.loose_steady(t_attn, t_ffn, 0.0, tau_attn, tau_ffn, L), info
        assert sum(r.stalls[nb:]) == 0.0
    else:
        assert not M.loose_steady(t_attn, t_ffn, 0.0, tau_attn, tau_ffn, L), info
    return info


if __name__ == "__main__":
    extra = int(sys.argv[3]) if len(sys.argv) > 3 else 0
    cal = len(sys.argv) > 4 and sys.argv[4] == "calibrate"
    print(f"pad {sys.argv[1]} T {sys.argv[2]}" + (f" after {extra} other streams" if extra else "") + ": " +
          run_case(int(sys.argv[1]), int(sys.argv[2]), extra, strict=len(sys.argv) <= 3 or cal, calibrate=cal), flush=True)
