"""Pins for the scheduler oracle (oracle/window_model.py): the values the paper
prints, and the event simulation against the paper's closed-form conditions."""
import os
import random

import pytest

from oracle import window_model as M

GOLD = os.path.join(os.path.dirname(__file__), "golden")
MiB, GiB = 2 ** 20, 2 ** 30


def _read(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].split()
        if len(line) >= 2:
            out[line[0]] = float(line[1])
    return out


def test_block_sizes_printed_in_the_paper():
    g = _read("paper_block_sizes.txt")
    h, a, b, s, v, p = 4096, 32, 32, 11008, 32000, 0.25           # Llama 2-7B, n = 4
    assert round(M.preprocess_params(h, v) * 4 / MiB) == g["preprocess_block"]
    assert round(M.attn_block_params(h, a, b, p) * 4 / MiB) == g["attention_block"]
    assert round(M.ffn_block_params(h, s, p) * 4 / MiB) == g["ffn_block"]
    assert round(M.postprocess_params(h, v) * 4 / MiB) == g["postprocess_block"]
    # Llama 2-70B: 80 layers x 8 shards of (attention + FFN block) + embedding + head
    h, a, b, s, v, p, L = 8192, 64, 8, 28672, 32000, 1 / 8, 80
    layer_shard = M.attn_block_params(h, a, b, p) + M.ffn_block_params(h, s, p)
    assert layer_shard == 106_971_136
    total = L * 8 * layer_shard + M.preprocess_params(h, v) + M.postprocess_params(h, v)
    assert round(total * 4 / GiB) == g["llama2_70b_total"]
    # the product's own shard-size function agrees with the paper's block formulas
    from paper_2410_00531_amd import configs
    assert configs.LLAMA2_70B_TP8.layer_shard_params() == layer_shard
    m = configs.LLAMA31_8B_TP4
    assert m.layer_shard_params() == M.attn_block_params(m.hidden, m.n_heads, m.n_kv_heads, 0.25) \
        + M.ffn_block_params(m.hidden, m.ffn, 0.25) == 54_534_144


def test_worked_example_of_the_steady_conditions():
    g = _read("paper_scheduler_example.txt")
    t = (g["t_attn"], g["t_ffn"], g["t_all_reduce"], g["tau_attn"], g["tau_ffn"])
    L, w = int(g["layers"]), int(g["window"])
    assert M.tight_steady(*t) == bool(g["tight_steady"])
    assert M.loose_steady(*t, L) == bool(g["loose_steady"])
    bal, first, second = M.loose_steady_branches(*t, L)
    assert bal and not first and second
    # the event simulation, which knows no formula: first block waits its own load,
    # the first FFN block waits tau_ffn - t_attn - t_ar = 5 ms (second branch), then nothing
    r = M.simulate(*t, n_layers=L, w=w, tokens=3)
    assert r.stalls[0] == g["tau_attn"]
    assert r.stalls[1] == g["tau_ffn"] - g["t_attn"] - g["t_all_reduce"]
    assert all(s == 0 for s in r.stalls[2:])
    # a window of one block cannot prefetch at all: every block waits for its whole load
    r1 = M.simulate(*t, n_layers=4, w=1)
    assert r1.stalls[2] > 0 and r1.stalls[3] > 0


def test_simulation_agrees_with_loose_condition_on_random_timings():
    """With room in the window the loader never idles.  Prop. 3's inequalities
    for l = 1..L speak about the FFN blocks of layers 1..L and the attention
    blocks of layers 2..L+1, i.e. blocks 1..2L (0-based) of a run of L+1 layers:
    'no block after the first FFN block waits' must coincide with the
    proposition exactly (integer timings, so no rounding)."""
    rnd = random.Random(0)
    seen = {True: 0, False: 0}
    for _ in range(4000):
        t_attn, t_ffn, t_ar = rnd.randint(1, 30), rnd.randint(1, 30), rnd.randint(0, 20)
        tau_attn, tau_ffn = rnd.randint(1, 40), rnd.randint(1, 40)
        L = rnd.randint(2, 12)
        args = (t_attn, t_ffn, t_ar, tau_attn, tau_ffn)
        r = M.simulate(*args, n_layers=L + 1, w=4 * L + 4)
        quiet = all(s == 0 for s in r.stalls[2:2 * L + 1])
        want = M.loose_steady(*args, L)
        assert quiet == want, (args, L)
        bal, first, second = M.loose_steady_branches(*args, L)
        if want and r.stalls[1] == 0:
            assert first                   # proof's case 1: the first FFN block did not wait
        if want and r.stalls[1] > 0:
            assert second and not first    # case 2: it waited tau_ffn - t_attn - t_ar
            assert r.stalls[1] == tau_ffn - t_attn - t_ar
        seen[want] += 1
    assert seen[True] > 200 and seen[False] > 200


def test_tight_implies_loose_and_no_stall():
    rnd = random.Random(1)
    n = 0
    for _ in range(3000):
        t = (rnd.randint(1, 30), rnd.randint(1, 30), rnd.randint(0, 20), rnd.randint(1, 40), rnd.randint(1, 40))
        if M.tight_steady(*t):
            n += 1
            assert M.loose_steady(*t, 16)
            r = M.simulate(*t, n_layers=16, w=2, tokens=2)     # even the smallest prefetching window
            assert all(s == 0 for s in r.stalls[1:]), t
    assert n > 100


def test_peak_memory_formula_matches_simulated_window():
    """Prop. 5 (worker, gamma = 1): when loads are fast the window is always
    full, and its worst content is floor(w/2) attention + floor((w+1)/2) FFN blocks."""
    h, a, b, s, p = 8192, 64, 8, 28672, 1 / 8
    sa, sf = M.attn_block_params(h, a, b, p), M.ffn_block_params(h, s, p)
    for w in range(1, 10):
        r = M.simulate(10, 10, 5, 1, 1, n_layers=12, w=w, tokens=2, size_attn=sa, size_ffn=sf)
        assert r.peak_blocks == w
        assert r.peak_resident == M.peak_worker_params(w, h, a, b, s, p)
    # a window of 8 blocks is 4 whole layer-shards
    assert M.peak_worker_params(8, h, a, b, s, p) == 4 * 106_971_136
    # master formula: continuity of its three cases and the worker part inside it
    v = 32000
    assert M.peak_master_params(1, h, v, a, b, s, p) == h * v + h
    assert M.peak_master_params(2, h, v, a, b, s, p) == 2 * h * v + h
    assert M.peak_master_params(4, h, v, a, b, s, p) == 2 * h * v + h + sa + sf
    assert M.peak_master_params(3, h, v, a, b, s, p, gamma=2.0) == 2 * (2 * h * v + h + sf)


def test_block_retention():
    """Prop. 6: keeping one FFN block of every T resident removes its load."""
    t = (11, 17, 14, 18, 30 + 20)            # a disk too slow for the plain window
    L = 12
    assert not M.loose_steady(*t, L)
    r = M.simulate(*t, n_layers=L, w=4)
    assert sum(r.stalls[2:]) > 0
    assert M.loose_steady_retention(*t, L, T=1)             # every FFN block resident
    r = M.simulate(*t, n_layers=L, w=4, retain_T=1)
    assert all(s == 0 for s in r.stalls[1:])
    # T large: only layer 1's FFN block is kept; cumulative deficit returns
    assert not M.loose_steady_retention(*t, L, T=100)
    # formula vs simulation on random integer timings (roomy window, so the loader never idles):
    # the two families for l = 1..L speak about blocks 1..2L of a run of L+1 layers
    rnd = random.Random(2)
    seen = {True: 0, False: 0}
    for _ in range(4000):
        tt = (rnd.randint(1, 30), rnd.randint(1, 30), rnd.randint(0, 20), rnd.randint(1, 40), rnd.randint(1, 60))
        T = rnd.randint(1, 4); L = rnd.randint(1, 10)
        sim = M.simulate(*tt, n_layers=L + 1, w=4 * L + 4, retain_T=T)
        quiet = all(s == 0 for s in sim.stalls[1:2 * L + 1])
        want = M.loose_steady_retention(*tt, L, T)
        assert quiet == want, (tt, T, L)
        seen[want] += 1
    assert seen[True] > 200 and seen[False] > 200


def test_hidden_fraction_definition():
    assert M.hidden_fraction(10.0, 10.0, 5.0) == 1.0
    assert M.hidden_fraction(15.0, 10.0, 5.0) == 0.0
    assert M.hidden_fraction(12.5, 10.0, 5.0) == 0.5


@pytest.mark.parametrize("h,a,b,s,v,p,L", [(4096, 32, 32, 11008, 32000, 0.25, 32),      # Llama 2-7B over 4 devices
                                             (8192, 64, 8, 28672, 32000, 0.125, 80)])    # Llama 2-70B over 8
def test_peak_memory_of_prop_5_is_the_largest_run_of_w_consecutive_blocks(h, a, b, s, v, p, L):
    """Prop. 5 by brute force: the master walks preprocess, (attention, FFN) x L, postprocess and on into the next
    token's preprocess; with w blocks resident its peak is the largest total of any w consecutive blocks of that
    cycle, the worker's the same over its (attention, FFN) x L cycle.  The closed forms must give exactly that."""
    attn, ffn = M.attn_block_params(h, a, b, p), M.ffn_block_params(h, s, p)
    master = [M.preprocess_params(h, v)] + [attn, ffn] * L + [M.postprocess_params(h, v)]
    worker = [attn, ffn] * L

    def brute(cycle, w):
        n = len(cycle)
        return max(sum(cycle[(i + k) % n] for k in range(w)) for i in range(n))

    for w in range(1, 9):
        assert M.peak_master_params(w, h, v, a, b, s, p) == brute(master, w), f"master, w = {w}"
        assert M.peak_worker_params(w, h, a, b, s, p) == brute(worker, w), f"worker, w = {w}"
