"""Oracle of the burst-parallel planner for graphs with branch/join blocks.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python floats (fp64), loops in the order
of the paper's Section 4.2, paragraph "Multi-chain graph reduction": the graph is a chain of main
layers; between two consecutive main layers there is either a direct edge or a block of parallel
branches that leave the first (the branching layer) and meet in the second (the joining layer).  A
block is reduced to one transition cost tr[g][h] (branching layer on g GPUs, joining layer on h), and
the chain algorithm of oracle/burst_plan.py then runs with tr in the place of comm.

Steps for one block, as the paragraph orders them:
  1. fix the GPU count g of the branching layer;
  2. run the chain search on every branch with its layer 0 pinned to g;
  3. for each GPU count h of the joining layer, take each branch's shortest time to reach it;
  4. the joining layer finds the critical (longest) branch and decides for every other branch whether
     it runs beside the critical one on GPUs of its own - only if moving its samples there and back
     neither lengthens the block nor exceeds the amplification limit - or after it;
  5. repeat for the next g.

Readings where the paragraph is silent (each also listed in the design notes):
  G1  Blocks do not nest; a branch is a (possibly empty) chain.  An empty branch is a skip connection:
      its time is its transfer join[g][h].
  G2  A branch's time to reach the joining layer on h GPUs is picked by the chain algorithm's own
      admission scan over the branch's last layer (the joining layer acting as layer L+1 with
      transition cost join[g'][h]).
  G3  Branches that do not run in parallel run one after another on the same GPUs: the block's time is
      the critical branch's time plus the times of the branches that were not moved aside.
  G4  A non-critical branch b may be moved aside when R_b + move_b[g][h] <= R_critical (the block
      does not get longer), where move_b is the caller's cost of taking the branch's samples to a new
      set of GPUs and back.  The new set has as many GPUs as the largest count on the branch's plan.
      Empty branches are never moved.  Ties for the critical branch go to the first.
  G5  Amplification of a joining layer counts the whole block: Amp = T * (h + GPUs of the sets that
      were added) / (one-GPU compute time of the joining layer and of all branch layers), T being the
      block's time plus the joining layer's comp and sync.  Candidates are tried in branch order; one
      is moved aside only if this amplification, with it moved, stays within the limit.
  G6  Inside a branch, Amp(l, g) = T[l][g] * g / comp(l, 1) as in the chain algorithm, and the pinned
      layer 0 is always admissible.

Pins (tests/test_graph_plan_pins.py): exhaustive enumeration of all assignments with no limit when no
branch can be moved (the block costs the sum of its branches) and when moving is free (the block costs
its longest branch); a block with a single branch against the chain planner on the flattened chain; a
hand-worked block with one branch moved aside and one not; the plan's own time recomputed from the
tables; an exhaustive lower bound with arbitrary move costs.
"""
import math

INF = math.inf


def _scan(cands, amp_limit):
    """The chain algorithm's admission scan: cands = [(index, amp, cost)] in GPU-count order."""
    best_amp, best_cost, pick = INF, INF, -1
    for idx, amp, cost in cands:
        if amp <= max(best_amp, amp_limit) and cost <= best_cost:
            best_cost, best_amp, pick = cost, min(best_amp, amp), idx
    return pick, best_cost


def search_branch(gpus, br, amp_limit, start):
    """Chain search over one branch with its layer 0 (the branching layer) pinned to gpus[start].
    Returns (S, T, H) with L_b + 1 rows; row 0 is the pinned start."""
    G, L = len(gpus), len(br["comp"])
    S = [[0.0 if b == start else INF for b in range(G)]] + [[INF] * G for _ in range(L)]
    T = [[0.0] * G] + [[INF] * G for _ in range(L)]
    H = [[-1] * G for _ in range(L + 1)]
    for i in range(1, L + 1):
        for a in range(G):
            if i == 1:
                cands = [(start, 0.0, br["comm"][0][start][a])]
            else:
                cands = [(b, T[i - 1][b] * gpus[b] / br["comp"][i - 2][0], S[i - 1][b] + br["comm"][i - 1][b][a]) for b in range(G)]
            pick, cost = _scan(cands, amp_limit)
            S[i][a] = cost + br["comp"][i - 1][a] + br["sync"][i - 1][a]
            T[i][a] = br["comm"][i - 1][pick][a] + br["comp"][i - 1][a] + br["sync"][i - 1][a]
            H[i][a] = pick
    return S, T, H


def branch_reach(gpus, br, amp_limit, start, S, T, H, a):
    """Shortest admitted time of the branch to reach the joining layer on gpus[a], the branch's plan
    (GPU-count indices) and the size of a GPU set that could hold it (reading G4)."""
    G, L = len(gpus), len(br["comp"])
    if L == 0:
        return br["join"][start][a], [], 0
    cands = [(b, T[L][b] * gpus[b] / br["comp"][L - 1][0], S[L][b] + br["join"][b][a]) for b in range(G)]
    pick, cost = _scan(cands, amp_limit)
    plan, b = [0] * L, pick
    for i in range(L, 0, -1):
        plan[i - 1] = b
        b = H[i][b]
    return cost, plan, max(gpus[p] for p in plan)


def reduce_block(gpus, branches, join_comp, join_sync, amp_limit):
    """tr[g][h] and the decisions behind it: info[g][h] = dict(critical, parallel, plans, extra, reach)."""
    G = len(gpus)
    one_gpu = join_comp[0] + sum(row[0] for br in branches for row in br["comp"])
    tr = [[INF] * G for _ in range(G)]
    info = [[None] * G for _ in range(G)]
    for g in range(G):
        searched = [search_branch(gpus, br, amp_limit, g) for br in branches]
        for h in range(G):
            reach = [branch_reach(gpus, br, amp_limit, g, *searched[k], h) for k, br in enumerate(branches)]
            times = [r[0] for r in reach]
            crit = max(range(len(branches)), key=lambda k: (times[k], -k))   # first of the longest
            t = sum(times)
            extra = 0
            parallel = [False] * len(branches)
            for k, br in enumerate(branches):
                if k == crit or not br["comp"] or not (times[k] + br["move"][g][h] <= times[crit]):
                    continue
                amp = (t - times[k] + join_comp[h] + join_sync[h]) * (gpus[h] + extra + reach[k][2]) / one_gpu
                if amp <= amp_limit:
                    t -= times[k]
                    extra += reach[k][2]
                    parallel[k] = True
            tr[g][h] = t
            info[g][h] = {"critical": crit, "parallel": parallel, "plans": [r[1] for r in reach], "extra": extra, "reach": times}
    return tr, info


def plan_graph(gpus, layers, amp_limit):
    """layers[i] = dict(comp=[G], sync=[G], comm=[G][G] or None, branches=[...] or []).  A layer with
    branches is the joining layer of a block whose branching layer is layer i-1 (i >= 1); a branch is
    dict(comp=[Lb][G], sync=[Lb][G], comm=[Lb][G][G], join=[G][G], move=[G][G]).
    Returns S, T (L+1 rows), the plan and the block decisions along it."""
    L, G = len(layers), len(gpus)
    assert gpus[0] == 1 and not layers[0].get("branches")
    S = [[0.0] * G] + [[INF] * G for _ in range(L)]
    T = [[0.0] * G] + [[INF] * G for _ in range(L)]
    H = [[-1] * G for _ in range(L + 1)]
    amp = [0.0] * G                      # Amp(i-1, .) for the scans of layer i
    blocks = [None] * L
    for i in range(1, L + 1):
        lay = layers[i - 1]
        if lay.get("branches"):
            tr, info = reduce_block(gpus, lay["branches"], lay["comp"], lay["sync"], amp_limit)
            blocks[i - 1] = info
            one_gpu = lay["comp"][0] + sum(row[0] for br in lay["branches"] for row in br["comp"])
        else:
            tr, info, one_gpu = lay["comm"], None, lay["comp"][0]
        new_amp = [0.0] * G
        for a in range(G):
            cands = [(b, amp[b], S[i - 1][b] + (tr[b][a] if tr is not None else 0.0)) for b in range(G)]
            pick, cost = _scan(cands, amp_limit)
            S[i][a] = cost + lay["comp"][a] + lay["sync"][a]
            T[i][a] = (tr[pick][a] if tr is not None else 0.0) + lay["comp"][a] + lay["sync"][a]
            H[i][a] = pick
            extra = info[pick][a]["extra"] if info is not None else 0
            new_amp[a] = T[i][a] * (gpus[a] + extra) / one_gpu
        amp = new_amp
    last, t = _scan([(a, amp[a], S[L][a]) for a in range(G)], amp_limit)
    plan, a = [0] * L, last
    for i in range(L, 0, -1):
        plan[i - 1] = a
        a = H[i][a]
    decisions = [blocks[i][plan[i - 1]][plan[i]] if blocks[i] is not None else None for i in range(L)]
    return {"S": S, "T": T, "H": H, "plan": plan, "gpus": [gpus[a] for a in plan], "time": t, "blocks": decisions}


def block_time(times, moves, can_move):
    """Reading G3/G4 with no amplification limit, for checks that recompute a plan's time: the longest
    branch plus every other branch that cannot be moved aside."""
    crit = max(range(len(times)), key=lambda k: (times[k], -k))
    return times[crit] + sum(t for k, t in enumerate(times) if k != crit and not (can_move[k] and t + moves[k] <= times[crit]))
