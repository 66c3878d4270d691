"""Oracle of the burst-parallel planner for a single chain of layers.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python floats (fp64), loops in the
order and notation of the paper's Section 4.2, Algorithm "Search Linear":

  S[i][g] = shortest time to complete L_1..L_i while using g GPUs for L_i
  T[i][g] = time spent on L_i while minimizing S[i][g]
  Amp(i, g) = T[i][g] * g / comp(i, 1)                      (GPU-sec amplification, Section 4.2)

The algorithm is a pruned shortest-path search, not an exact constrained optimum, so this file takes
its steps as printed.  Inputs are tables: comp[i][a] for layer i (0-based here, L_{i+1} in the paper)
at GPU count gpus[a]; comm[i][b][a] = comm_{(i-1, gpus[b]) -> (i, gpus[a])} for i >= 1 (comm[0] is the
transition into the first layer); sync[i][a].

Readings where the text is silent (each also listed in the design notes):
  * "g in [1, G]" ranges over a caller-given ascending list of GPU counts whose first entry is 1
    (needed for comp(i, 1)); the evaluation restricts it to powers of two.
  * Layer 0 does not exist: S[0][g] = 0 as printed, Amp(0, h) = 0 (always admissible), and the
    transition into L_1 is whatever comm[0] holds (zeros: input loading is not modelled).
  * The back-trace needs the h that produced bestS; it is recorded next to S and T.
  * The last layer's g is picked with the same admission rule the loop applies to a predecessor
    (a virtual layer L+1 with zero transition cost): scan g in order, admit when
    Amp(L, g) <= max(bestAmp, AmpLimit) and S[L][g] <= bestS.

The closed-form cost model (Section 4.1: payload divided by per-GPU bandwidth plus a propagation
delay, full bisection) is in comm_model / sync_model; the payload split between GPU sets is a
reading, stated at each function.

Pins (tests/test_planner_pins.py): exhaustive enumeration of all assignments with AmpLimit = inf,
a hand-worked two-layer example, Amp(i,1) = 1 without communication, perfectly linear scaling,
path-sum consistency of the back-trace, the all-ones plan as an upper bound.
"""
import math

INF = math.inf


def search_linear(gpus, comp, comm, sync, amp_limit):
    """Algorithm "Search Linear".  Returns (S, T, H): tables of L+1 rows (row 0 = the printed
    initialisation) and the predecessor index H[i][a] (index into gpus) behind S[i][a]."""
    L, G = len(comp), len(gpus)
    assert gpus[0] == 1 and all(gpus[a] < gpus[a + 1] for a in range(G - 1))
    S = [[0.0] * G] + [[INF] * G for _ in range(L)]
    T = [[0.0] * G] + [[INF] * G for _ in range(L)]
    H = [[-1] * G for _ in range(L + 1)]

    def amp(i, b):   # Amp(i, gpus[b]); layer 0 is always admissible
        if i == 0:
            return 0.0
        return T[i][b] * gpus[b] / comp[i - 1][0]

    for i in range(1, L + 1):
        for a in range(G):
            best_amp, best_s, best_t, best_h = INF, INF, INF, -1
            for b in range(G):
                c = comm[i - 1][b][a]
                if amp(i - 1, b) <= max(best_amp, amp_limit) and S[i - 1][b] + c <= best_s:
                    best_s = S[i - 1][b] + c
                    best_t = c
                    best_amp = min(best_amp, amp(i - 1, b))
                    best_h = b
            S[i][a] = best_s + comp[i - 1][a] + sync[i - 1][a]
            T[i][a] = best_t + comp[i - 1][a] + sync[i - 1][a]
            H[i][a] = best_h
    return S, T, H


def amplification(gpus, comp, T):
    """Amp(i, g) for i = 1..L as a list of rows (row i-1 for layer i)."""
    return [[T[i][a] * gpus[a] / comp[i - 1][0] for a in range(len(gpus))] for i in range(1, len(comp) + 1)]


def backtrace(gpus, comp, S, T, H, amp_limit):
    """GPU-count index per layer (length L) and the iteration time S[L][g_L]."""
    L, G = len(comp), len(gpus)
    best_amp, best_s, last = INF, INF, -1
    for a in range(G):
        am = T[L][a] * gpus[a] / comp[L - 1][0]
        if am <= max(best_amp, amp_limit) and S[L][a] <= best_s:
            best_s, best_amp, last = S[L][a], min(best_amp, am), a
    plan = [0] * L
    a = last
    for i in range(L, 0, -1):
        plan[i - 1] = a
        a = H[i][a]
    return plan, best_s


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
