"""Oracle of the burst-parallel planner for a single chain of layers.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python floats (fp64).  What it computes is
the dynamic programme of the paper's Section 4.2, Algorithm "Search Linear", over two tables indexed by
(layer, GPU count):

  S[i][g]   the earliest finish of layer i when that layer runs on g GPUs, over the predecessor
            choices the search admits;
  T[i][g]   the part of that finish time that belongs to layer i alone: the transition into it plus
            its compute and gradient synchronisation;
  Amp(i, g) = T[i][g] * g / comp(i, 1), how many single-GPU seconds the layer costs per second it would
            take on one GPU (the paper's GPU-sec amplification).

The search is pruned (a predecessor is dropped once its amplification is over the limit and over the best
admitted before it), so it is not an exact constrained optimum and cannot be replaced by a textbook
shortest path; this file therefore performs the search's decisions in the paper's scan order (GPU counts
ascending), organised as one admission helper plus a table fill.  Inputs are tables: comp[i][a] for layer
i (0-based here) at GPU count gpus[a]; comm[i][b][a] = cost of going from layer i-1 on gpus[b] to layer i
on gpus[a] (comm[0] leads into the first layer); sync[i][a].

Readings where the text is silent (each also listed in the design notes):
  * GPU counts are a caller-given ascending list whose first entry is 1 (comp(i, 1) is needed); the
    evaluation restricts it to powers of two.
  * There is no layer 0: its row of S is zero and it is always admissible (amplification 0); the
    transition into the first layer is whatever comm[0] holds (zeros: input loading is not modelled).
  * The admission test compares against max(best amplification admitted so far, limit) with "best so
    far" starting at infinity: the first candidate scanned always passes; ties in arrival time go to
    the later candidate.
  * The back-trace needs the predecessor behind each S entry; it is recorded in a third table.
  * The last layer's GPU count is picked by the same admission helper (a virtual successor with zero
    transition cost).

The closed-form cost model (Section 4.1: payload divided by per-GPU bandwidth plus a propagation
delay, full bisection) is in comm_time / sync_time; the payload split between GPU sets is a
reading, stated at each function.

Pins (tests/test_planner_pins.py): exhaustive enumeration of all assignments with no limit,
a hand-worked two-layer example, Amp(i,1) = 1 without communication, perfectly linear scaling,
path-sum consistency of the back-trace, the all-ones plan as an upper bound.
"""
import math

INF = math.inf


def admit(candidates, amp_limit):
    """One admission scan.  candidates: (amplification, arrival time, payload) triples in ascending
    GPU-count order.  A candidate is taken when its amplification is within the limit or no worse than
    the smallest one taken so far, and its arrival is not later than the current best.
    Returns (best arrival, payload of the candidate behind it), payload None if nothing was scanned."""
    lowest_amp, best_arrival, chosen = INF, INF, None
    for amp, arrival, payload in candidates:
        if amp > max(lowest_amp, amp_limit) or arrival > best_arrival:
            continue
        best_arrival, chosen = arrival, payload
        lowest_amp = min(lowest_amp, amp)
    return best_arrival, chosen


def search_linear(gpus, comp, comm, sync, amp_limit):
    """Fills S, T (L+1 rows; row 0 is the start state) and H, the index into gpus of the predecessor
    count behind each S entry."""
    L, G = len(comp), len(gpus)
    assert gpus[0] == 1 and all(gpus[a] < gpus[a + 1] for a in range(G - 1))
    S = [[0.0] * G] + [[INF] * G for _ in range(L)]
    T = [[0.0] * G] + [[INF] * G for _ in range(L)]
    H = [[-1] * G for _ in range(L + 1)]
    for layer in range(1, L + 1):
        own = comp[layer - 1]
        # amplification of every predecessor state; the start state costs nothing
        prev_amp = [0.0 if layer == 1 else T[layer - 1][b] * gpus[b] / comp[layer - 2][0] for b in range(G)]
        for a in range(G):
            hop = [comm[layer - 1][b][a] for b in range(G)]
            arrival, b = admit([(prev_amp[b], S[layer - 1][b] + hop[b], b) for b in range(G)], amp_limit)
            # summed left to right, as the algorithm writes the two sums
            S[layer][a] = arrival + own[a] + sync[layer - 1][a]
            T[layer][a] = (hop[b] if b is not None else INF) + own[a] + sync[layer - 1][a]
            H[layer][a] = b if b is not None else -1
    return S, T, H


def amplification(gpus, comp, T):
    """Amp(i, g) for i = 1..L as a list of rows (row i-1 for layer i)."""
    return [[T[i][a] * gpus[a] / comp[i - 1][0] for a in range(len(gpus))] for i in range(1, len(comp) + 1)]


def backtrace(gpus, comp, S, T, H, amp_limit):
    """GPU-count index per layer (length L) and the iteration time S[L][g_L]."""
    L, G = len(comp), len(gpus)
    final = [(T[L][a] * gpus[a] / comp[L - 1][0], S[L][a], a) for a in range(G)]
    total, a = admit(final, amp_limit)
    plan = [0] * L
    for layer in range(L, 0, -1):
        plan[layer - 1] = a
        a = H[layer][a]
    return plan, total


def plan_chain(gpus, comp, comm, sync, amp_limit):
    S, T, H = search_linear(gpus, comp, comm, sync, amp_limit)
    plan, t = backtrace(gpus, comp, S, T, H, amp_limit)
    return {"S": S, "T": T, "H": H, "plan": plan, "gpus": [gpus[a] for a in plan], "time": t}


# ---- closed-form cost model (Section 4.1) ---------------------------------------------------------
def comm_time(act_bytes, g, h, bandwidth, delay):
    """comm_{(i,g)->(j,h)}: activations of the global batch (act_bytes in total) move forward and their
    gradients move back when the GPU count changes between two layers.  Reading: samples are spread
    evenly, a GPU of the smaller set holds 1/min(g,h) of them and keeps 1/max(g,h), so it sends (or
    receives) act_bytes * (1/min - 1/max); that per-GPU payload over the per-GPU bandwidth plus the
    propagation delay, once per direction."""
    if g == h:
        return 0.0
    lo, hi = (g, h) if g < h else (h, g)
    payload = act_bytes * (1.0 / lo - 1.0 / hi)
    return 2.0 * (payload / bandwidth + delay)


def sync_time(param_bytes, g, bandwidth, delay):
    """sync_{(i,g)}: gradient synchronisation of one layer over g GPUs, not overlapped with the backward
    pass.  Reading: a reduce-scatter followed by an all-gather, each moving param_bytes * (g-1)/g per
    GPU, each paying the propagation delay once."""
    if g == 1:
        return 0.0
    return 2.0 * (param_bytes * (g - 1.0) / g / bandwidth + delay)


def cost_tables(gpus, act_bytes, param_bytes, bandwidth, delay):
    """comm[i][b][a] and sync[i][a] from payload sizes: act_bytes[i] = bytes entering layer i (i = 0 is
    the network input and costs nothing: it is loaded where it is needed), param_bytes[i] = gradient
    bytes of layer i."""
    L, G = len(param_bytes), len(gpus)
    comm = [[[0.0 if i == 0 else comm_time(act_bytes[i], gpus[b], gpus[a], bandwidth, delay) for a in range(G)]
             for b in range(G)] for i in range(L)]
    sync = [[sync_time(param_bytes[i], gpus[a], bandwidth, delay) for a in range(G)] for i in range(L)]
    return comm, sync
