"""The window's slot state machine (prefetch / acquire / release, ring slots, retention, the file tier's
loader thread) on the library's host model of queues, events and copies -- no GPU.

Two things are checked.  Ordering: the model executes what the window queued in seeded random orders that
respect queue order and event waits only; every "kernel" must still see the bytes of the block it acquired
(a copy that overtakes a reader, or a reader that overtakes its copy, gives a wrong hash in some order).
Timing: with the paper's notation (t_attn, t_ffn, t_all-reduce, tau_attn, tau_ffn; Sec. 3.3, Prop. 3-6) the
model's clocks must reproduce, block by block, what the scheduler oracle's event simulation predicts, and the
slots a window of w blocks needs must be the peak memory of Prop. 5."""
import ctypes as C

import numpy as np
import pytest

from oracle import window_model as M
from paper_2410_00531_amd import binding as B
from paper_2410_00531_amd import configs, synth


def _addr(a: np.ndarray) -> int:
    return a.ctypes.data


def _make_blocks(rng, L, n_attn, n_ffn):
    """Blocks 2l / 2l+1: attention / FFN block of layer l, distinct random bytes."""
    return [rng.integers(0, 256, size=(n_ffn if b % 2 else n_attn), dtype=np.uint8) for b in range(2 * L)]


def _drive(win, sim, stream, L, n_tokens, w, block_ptr_bytes, costs, release_first=False):
    """The scheduler's loop of Sec. 3.3 over blocks 0 .. 2L-1, n_tokens times: w blocks are requested ahead,
    every release is followed by the next request.  costs = (t_attn, t_ffn, t_ar).  Returns the per-block
    (hash cell, start cell, block index) of the reads."""
    total = 2 * L * n_tokens
    issued = 0

    def prefetch_next():
        nonlocal issued
        if issued < total:
            win.prefetch(issued % (2 * L))
            issued += 1

    for _ in range(w):
        prefetch_next()
    reads = []
    for i in range(total):
        b = i % (2 * L)
        ptr = win.acquire(b, stream)
        nbytes = block_ptr_bytes[b]
        if release_first:                       # a caller's mistake: the slot is given back before its reader is queued
            win.release(b, stream)
            prefetch_next()
            cell, start = sim.read(stream, ptr, nbytes, costs[b % 2])
        else:
            cell, start = sim.read(stream, ptr, nbytes, costs[b % 2])
            win.release(b, stream)
            prefetch_next()
        sim.read(stream, 0, 0, costs[2])        # the all-reduce after every block
        reads.append((cell, start, b))
    return reads


def _block_window(sim, blocks, L, w, T, n_attn, n_ffn):
    retained = {2 * l + 1 for l in range(L) if T and l % T == 0}
    homes = {b: np.zeros(n_ffn, np.uint8) for b in retained}
    slots_a = np.zeros((w // 2) * n_attn, np.uint8)
    slots_f = np.zeros(max(1, (w + 1) // 2) * n_ffn, np.uint8)
    spec = [(_addr(blocks[b]), blocks[b].nbytes, b % 2, _addr(homes[b]) if b in homes else None) for b in range(2 * L)]
    win = B.Window.from_blocks(spec, [(_addr(slots_a), n_attn, w // 2), (_addr(slots_f), n_ffn, max(1, (w + 1) // 2))],
                               sim=sim)
    return win, (homes, slots_a, slots_f), retained


@pytest.mark.parametrize("L,w,T", [(4, 2, 0), (5, 4, 0), (6, 4, 2), (7, 6, 3), (3, 2, 1)])
def test_every_reader_sees_its_block_in_every_order(L, w, T):
    n_attn, n_ffn = 96, 160
    rng = np.random.default_rng(L * 100 + w * 10 + T)
    blocks = _make_blocks(rng, L, n_attn, n_ffn)
    want = [B.Sim.hash(_addr(b), b.nbytes) for b in blocks]
    for seed in range(40):
        sim = B.Sim(seed)
        stream = sim.stream()
        win, keep, _ = _block_window(sim, blocks, L, w, T, n_attn, n_ffn)
        reads = _drive(win, sim, stream, L, 3, w, [b.nbytes for b in blocks], (1.0, 1.0, 0.0))
        sim.run()
        for cell, _, b in reads:
            assert cell.value == want[b], f"seed {seed}: the reader of block {b} saw other bytes"
        win.destroy()
        sim.destroy()


def test_the_model_catches_a_slot_released_before_its_reader_is_queued():
    """The detector has teeth: with release (and the next request) ahead of the read, the next tenant's copy
    is no longer ordered behind the reader, and some order shows it."""
    L, w, n_attn, n_ffn = 4, 2, 96, 160
    rng = np.random.default_rng(1)
    blocks = _make_blocks(rng, L, n_attn, n_ffn)
    want = [B.Sim.hash(_addr(b), b.nbytes) for b in blocks]
    wrong = 0
    for seed in range(40):
        sim = B.Sim(seed)
        stream = sim.stream()
        win, keep, _ = _block_window(sim, blocks, L, w, 0, n_attn, n_ffn)
        reads = _drive(win, sim, stream, L, 3, w, [b.nbytes for b in blocks], (1.0, 1.0, 0.0), release_first=True)
        sim.run()
        wrong += sum(cell.value != want[b] for cell, _, b in reads)
        win.destroy()
        sim.destroy()
    assert wrong > 0


def test_layer_window_ring_and_wraparound_on_the_model():
    """tpi_window_create's ring (whole layers) is the block window with one class: drive it through the same
    model via one-class blocks, five layers through three slots, four tokens."""
    L, W, n = 5, 3, 200
    rng = np.random.default_rng(2)
    layers = [rng.integers(0, 256, size=n, dtype=np.uint8) for _ in range(L)]
    want = [B.Sim.hash(_addr(b), n) for b in layers]
    for seed in range(20):
        sim = B.Sim(seed)
        stream = sim.stream()
        slots = np.zeros(W * n, np.uint8)
        win = B.Window.from_blocks([(_addr(b), n, 0, None) for b in layers], [(_addr(slots), n, W)], sim=sim)
        issued = 0
        for _ in range(W):
            win.prefetch(issued % L); issued += 1
        reads = []
        for i in range(4 * L):
            l = i % L
            ptr = win.acquire(l, stream)
            assert ptr == _addr(slots) + (i % W) * n          # ring order
            reads.append((sim.read(stream, ptr, n, 1.0)[0], l))
            win.release(l, stream)
            if issued < 4 * L:
                win.prefetch(issued % L); issued += 1
        sim.run()
        assert all(c.value == want[l] for c, l in reads)
        ms, copied = win.copy_stats()
        assert copied == 4 * L * n and ms > 0
        win.destroy(); sim.destroy()


def test_file_tier_on_the_model(tmp_path):
    """The loader thread, its staging ring and the parallel readers, against the same model."""
    L, w, T, n_attn, n_ffn = 4, 2, 2, 4096, 3 << 19           # FFN blocks above 1 MiB: several reader threads
    rng = np.random.default_rng(3)
    blocks = _make_blocks(rng, L, n_attn, n_ffn)
    want = [B.Sim.hash(_addr(b), b.nbytes) for b in blocks]
    path = str(tmp_path / "stack.bin")
    offs = []
    with open(path, "wb") as f:
        for b in blocks:
            offs.append(f.tell()); f.write(b.tobytes())
    for seed in range(6):
        sim = B.Sim(seed)
        stream = sim.stream()
        retained = {2 * l + 1 for l in range(L) if l % T == 0}
        homes = {b: np.zeros(n_ffn, np.uint8) for b in retained}
        slots_a = np.zeros(n_attn, np.uint8); slots_f = np.zeros(n_ffn, np.uint8)
        spec = [(path, offs[b], blocks[b].nbytes, b % 2, _addr(homes[b]) if b in homes else None) for b in range(2 * L)]
        win = B.Window.from_files(spec, [(_addr(slots_a), n_attn, 1), (_addr(slots_f), n_ffn, 1)], n_staging=2,
                                  n_readers=3, sim=sim)
        reads = _drive(win, sim, stream, L, 3, w, [b.nbytes for b in blocks], (1.0, 1.0, 0.0))
        _, copied = win.copy_stats()                          # waits for the loader to have queued everything
        sim.run()
        per_token = L * n_attn + (L - len(retained)) * n_ffn
        assert copied == 3 * per_token + len(retained) * n_ffn
        for cell, _, b in reads:
            assert cell.value == want[b], f"seed {seed}: the reader of block {b} saw other bytes"
        win.destroy(); sim.destroy()


def _timed_run(L, w, T, t, tokens):
    """Drives the block window on the model with the paper's five times; tau = bytes / rate exactly."""
    t_attn, t_ffn, t_ar, tau_attn, tau_ffn = t
    rate = 16.0                                               # bytes per model millisecond
    n_attn, n_ffn = int(tau_attn * rate), int(tau_ffn * rate)
    rng = np.random.default_rng(4)
    blocks = _make_blocks(rng, L, n_attn, n_ffn)
    sim = B.Sim(11)
    sim.set_copy_rate(rate)
    stream = sim.stream()
    win, keep, retained = _block_window(sim, blocks, L, w, T, n_attn, n_ffn)
    reads = _drive(win, sim, stream, L, tokens, w, [b.nbytes for b in blocks], (t_attn, t_ffn, t_ar))
    sim.run()
    starts = [s.value for _, s, _ in reads]
    finish = sim.stream_time(stream)
    win.destroy(); sim.destroy()
    return starts, finish


@pytest.mark.parametrize("t", [(11.0, 17.0, 14.0, 18.0, 30.0),      # the paper's worked example (Sec. 3.3)
                               (5.0, 9.0, 1.0, 12.0, 20.0),        # copy-bound: every block waits
                               (20.0, 30.0, 2.0, 4.0, 9.0),        # compute-bound: only the first block waits
                               (7.0, 3.0, 0.0, 6.0, 11.0)])
@pytest.mark.parametrize("L,w", [(4, 2), (6, 4), (5, 6)])
def test_window_timing_equals_the_scheduler_oracle(t, L, w):
    """Block by block, the start times the window produces on the model equal the oracle's event simulation
    (which knows nothing of slots, rings or events), and so do the stalls that Prop. 3 / 4 speak about."""
    tokens = 3
    starts, finish = _timed_run(L, w, 0, t, tokens)
    r = M.simulate(*t, n_layers=L, w=w, tokens=tokens)
    assert starts == r.start
    assert finish == r.finish
    # Prop. 4 (tight steady condition) on these times: if it holds nothing waits after the first window
    if M.tight_steady(*t):
        assert all(s == 0 for s in r.stalls[w:])


@pytest.mark.parametrize("T", [1, 2, 3])
def test_retention_timing_in_the_steady_state_equals_the_oracle(T):
    """Prop. 6: with one FFN block of every T resident the copy-bound token gets shorter.  The window loads a
    retained block once, on first use, the oracle assumes it resident from the start; once all are in, a
    token takes the same time in both."""
    t, L, w = (5.0, 9.0, 1.0, 12.0, 20.0), 6, 4
    tokens = 5
    starts, _ = _timed_run(L, w, T, t, tokens)
    r = M.simulate(*t, n_layers=L, w=w, tokens=tokens, retain_T=T)
    nb = 2 * L
    assert starts[4 * nb] - starts[3 * nb] == r.start[4 * nb] - r.start[3 * nb]
    # and retention pays: the same window without it is slower per token
    plain = M.simulate(*t, n_layers=L, w=w, tokens=tokens)
    assert r.start[4 * nb] - r.start[3 * nb] < plain.start[4 * nb] - plain.start[3 * nb]


@pytest.mark.parametrize("w", [2, 4, 6, 8])
def test_slots_of_a_window_are_the_peak_memory_of_prop_5(w):
    """A window of w blocks (w even) is w/2 attention slots + w/2 FFN slots: in parameters exactly the worker's
    peak of Prop. 5 at the 70B-shaped 8-way shard, and the oracle's event simulation never has more resident."""
    m = configs.LLAMA2_70B_TP8
    shapes = synth.shard_tensor_shapes(m.hidden, m.nq_local, m.nkv_local, m.head_dim, m.ffn_local)
    n_attn = sum(int(np.prod(shapes[k])) for k in ("attn_norm", "w_qkv", "w_o"))
    n_ffn = sum(int(np.prod(shapes[k])) for k in ("ffn_norm", "w_gate", "w_up", "w_down"))
    slots = (w // 2) * n_attn + (w // 2) * n_ffn
    assert slots == M.peak_worker_params(w, m.hidden, m.n_heads, m.n_kv_heads, m.ffn, 1.0 / m.n_shards)
    r = M.simulate(1.0, 1.0, 0.0, 5.0, 9.0, n_layers=8, w=w, tokens=2, size_attn=n_attn, size_ffn=n_ffn)
    assert r.peak_resident <= slots and r.peak_blocks <= w


def test_sim_argument_errors():
    sim = B.Sim(0)
    other = B.Sim(1)
    a = np.zeros(16, np.uint8)
    with pytest.raises(B.TpiError) as ei:
        sim.read(other.stream(), _addr(a), 16)
    assert ei.value.code == B.TPI_EINVAL
    assert B.lib().tpi_sim_run(None) == B.TPI_EINVAL
    assert B.lib().tpi_window_create_blocks_sim(C.byref(C.c_void_p()), None, 1, None, 1, None) == B.TPI_EINVAL
    sim.destroy(); other.destroy()
