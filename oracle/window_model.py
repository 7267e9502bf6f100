"""TEST INFRASTRUCTURE -- not part of the product path.

Host-side oracle for the sliding-window memory scheduler of TPI-LLM
(Sec. 3.3; Prop. 3-6; appendix proofs of Prop. 3, 5 and 6; appendix
parameter-count table).  Two independent things live here so that one can pin
the other:

  * the closed forms the paper prints (block parameter counts, steady
    conditions, peak memory), written out as formulas;
  * a discrete-event simulation of the scheduler itself (a loader that fetches
    blocks one after another in execution order while at most ``w`` blocks are
    resident, and a compute thread that waits for a block, runs it, releases
    it, then spends one all-reduce), which knows none of those formulas.

Blocks alternate attention, FFN, attention, ... over the layers of one token
and wrap to the next token's first attention block.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional


# ----------------------------------------------------------------------------
# Closed forms printed in the paper
# ----------------------------------------------------------------------------

def attn_block_params(h: int, a: int, b: int, p: float) -> float:
    """Attention block: 2(a+b) h^2 p / a + h  (W_Q, W_O: h^2 p each; W_K, W_V:
    (b/a) h^2 p each; one norm gain).  Appendix parameter-count table."""
    return 2.0 * (a + b) * h * h * p / a + h


def ffn_block_params(h: int, s: int, p: float) -> float:
    """FFN block: 3 h s p + h (gate, up, down and one norm gain)."""
    return 3.0 * h * s * p + h


def preprocess_params(h: int, v: int) -> float:
    return float(h) * v


def postprocess_params(h: int, v: int) -> float:
    return float(h) * v + h


def peak_worker_params(w: int, h: int, a: int, b: int, s: int, p: float, gamma: float = 1.0) -> float:
    """Prop. 5, worker: gamma * (floor(w/2) attn + floor((w+1)/2) ffn)."""
    return gamma * ((w // 2) * attn_block_params(h, a, b, p)
                    + ((w + 1) // 2) * ffn_block_params(h, s, p))


def peak_master_params(w: int, h: int, v: int, a: int, b: int, s: int, p: float,
                       gamma: float = 1.0) -> float:
    """Prop. 5, master."""
    if w == 1:
        return gamma * (h * v + h)
    if w == 2:
        return gamma * (2 * h * v + h)
    return gamma * (2 * h * v + h + ((w - 2) // 2) * attn_block_params(h, a, b, p)
                    + ((w - 1) // 2) * ffn_block_params(h, s, p))


def tight_steady(t_attn, t_ffn, t_ar, tau_attn, tau_ffn) -> bool:
    """Prop. 4."""
    return (t_attn + t_ar >= tau_ffn) and (t_ffn + t_ar >= tau_attn)


def loose_steady(t_attn, t_ffn, t_ar, tau_attn, tau_ffn, L: int) -> bool:
    """Prop. 3: the per-layer balance and one of the two cumulative branches."""
    if not (t_attn + t_ffn + 2 * t_ar >= tau_ffn + tau_attn):
        return False
    first = all(l * t_attn + (l - 1) * t_ffn + (2 * l - 1) * t_ar
                >= l * tau_ffn + (l - 1) * tau_attn for l in range(1, L + 1))
    second = all((l - 1) * t_attn + l * t_ffn + (2 * l - 1) * t_ar
                 >= (l - 1) * tau_ffn + l * tau_attn for l in range(1, L + 1))
    return first or second


def loose_steady_branches(t_attn, t_ffn, t_ar, tau_attn, tau_ffn, L: int):
    """(balance, first branch, second branch) of Prop. 3, separately."""
    bal = t_attn + t_ffn + 2 * t_ar >= tau_ffn + tau_attn
    first = all(l * t_attn + (l - 1) * t_ffn + (2 * l - 1) * t_ar
                >= l * tau_ffn + (l - 1) * tau_attn for l in range(1, L + 1))
    second = all((l - 1) * t_attn + l * t_ffn + (2 * l - 1) * t_ar
                 >= (l - 1) * tau_ffn + l * tau_attn for l in range(1, L + 1))
    return bal, first, second


def loose_steady_retention(t_attn, t_ffn, t_ar, tau_attn, tau_ffn, L: int, T: int) -> bool:
    """Prop. 6: one FFN block of every T stays resident (l = 1 + kT)."""
    for l in range(1, L + 1):
        kept = math.ceil(l / T)
        if not (l * t_attn + l * t_ffn + 2 * l * t_ar >= (l - kept) * tau_ffn + l * tau_attn):
            return False
        if not (l * t_attn + (l - 1) * t_ffn + (2 * l - 1) * t_ar
                >= (l - kept) * tau_ffn + (l - 1) * tau_attn):
            return False
    return True


# ----------------------------------------------------------------------------
# Discrete-event simulation of the scheduler
# ----------------------------------------------------------------------------

@dataclass
class SimResult:
    stalls: List[float]          # per block: time compute waited for its weights
    start: List[float]           # per block: compute start
    load_done: List[float]       # per block: time its weights were resident
    finish: float                # end of the last all-reduce
    peak_resident: float         # max over time of the sizes of resident blocks
    peak_blocks: int


def simulate(t_attn, t_ffn, t_ar, tau_attn, tau_ffn, n_layers: int, w: int, tokens: int = 1,
             size_attn: float = 1.0, size_ffn: float = 1.0,
             retain_T: Optional[int] = None) -> SimResult:
    """Event simulation of the scheduler thread and the compute thread.

    Loader: fetches blocks in execution order, one at a time; it may begin
    block i only once fewer than ``w`` streamed blocks are resident (resident =
    fetch begun and not yet released).  Compute: block i starts when the
    previous block's all-reduce has ended and block i is loaded; the block is
    released when its computation ends (the context manager's exit); one
    all-reduce follows every block.  With ``retain_T`` the FFN blocks of layers
    1, 1+T, 1+2T, ... (1-based) are pinned outside the window and cost no load.
    """
    assert w >= 1 and n_layers >= 1 and tokens >= 1
    nb = 2 * n_layers * tokens
    kind = [i % 2 for i in range(nb)]                      # 0 attention, 1 FFN
    layer1 = [(i // 2) % n_layers + 1 for i in range(nb)]  # 1-based layer of block i
    retained = [bool(retain_T) and kind[i] == 1 and (layer1[i] - 1) % retain_T == 0
                for i in range(nb)]
    tau = [0.0 if retained[i] else (tau_ffn if kind[i] else tau_attn) for i in range(nb)]
    tc = [t_ffn if kind[i] else t_attn for i in range(nb)]
    size = [size_ffn if kind[i] else size_attn for i in range(nb)]

    load_begin = [0.0] * nb
    load_done = [0.0] * nb
    start = [0.0] * nb
    release = [0.0] * nb
    stalls = [0.0] * nb
    streamed = [i for i in range(nb) if not retained[i]]
    order = {b: k for k, b in enumerate(streamed)}         # position among streamed blocks

    loader_free = 0.0
    ready = 0.0                                            # compute thread free at
    # The loader's decision for block i depends only on releases of earlier
    # blocks, and compute of block i only on load_done[i]: one forward pass.
    for i in range(nb):
        if retained[i]:
            load_begin[i] = load_done[i] = 0.0
        else:
            k = order[i]
            gate = release[streamed[k - w]] if k >= w else 0.0
            load_begin[i] = max(loader_free, gate)
            load_done[i] = load_begin[i] + tau[i]
            loader_free = load_done[i]
        start[i] = max(ready, load_done[i])
        stalls[i] = start[i] - ready
        release[i] = start[i] + tc[i]
        ready = release[i] + t_ar

    # peak of resident streamed bytes: sweep the begin / release events
    ev = []
    for i in streamed:
        ev.append((load_begin[i], 1, size[i]))
        ev.append((release[i], 0, -size[i]))               # releases first at equal times
    ev.sort(key=lambda e: (e[0], e[1]))
    cur = 0.0; peak = 0.0; nblk = 0; peak_blk = 0
    for _, _, s in ev:
        cur += s; nblk += 1 if s > 0 else -1
        peak = max(peak, cur); peak_blk = max(peak_blk, nblk)
    return SimResult(stalls, start, load_done, ready, peak, peak_blk)


def hidden_fraction(t_token_windowed: float, t_token_resident: float, copy_time: float) -> float:
    """1 - (extra time of the windowed run) / (total copy time)."""
    if copy_time <= 0:
        return 1.0
    return 1.0 - (t_token_windowed - t_token_resident) / copy_time
