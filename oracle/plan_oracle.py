"""Plan-side oracle (TEST INFRASTRUCTURE ONLY): operation counts, the size of the joint
fusion/MP search space, exhaustive enumeration of fusion schemes, and the greedy pass of the
paper's Algorithm 1, written from the paper's equations and prose.  Shares no code with the GPU
library's planner.
"""
import itertools
import math

CONV_LIKE = ("conv", "dwconv", "fc")


# --------------------------------------------------------------------------------------------
# Operation counts (Eq. 1, Eq. 2) and operational intensity (Eq. 3)
# --------------------------------------------------------------------------------------------

def mac_count(L, out_h, out_w, batch=1):
    """Multiply-accumulates of one layer.  Convolution: Hout*Wout*Hk*Wk*Cin*Cout (per group:
    Cin/groups inputs per output channel); FC: M*K*N with M = batch.  Pooling counts zero."""
    if L["op"] == "conv":
        return batch * out_h * out_w * L["kh"] * L["kw"] * L["cin"] * L["cout"]
    if L["op"] == "dwconv":
        return batch * out_h * out_w * L["kh"] * L["kw"] * L["cout"]
    if L["op"] == "fc":
        return batch * L["cin"] * L["cout"]
    return 0


def op_count(L, out_h, out_w, batch=1):
    """Eq. 1 / Eq. 2: operations = 2 x MAC."""
    return 2 * mac_count(L, out_h, out_w, batch)


def intensity(ops, tensor_bytes):
    """Eq. 3: operations divided by the summed size of the tensors touched."""
    return ops / float(sum(tensor_bytes))


# --------------------------------------------------------------------------------------------
# Search space (Sec. III-C, Eq. 4)
# --------------------------------------------------------------------------------------------

def space_eq4(n, n_mp=32):
    """Eq. 4 as printed: sum over i = 1..n-1 cut points of n_mp^(i+1) * C(n-1, i)."""
    return sum(n_mp ** (i + 1) * math.comb(n - 1, i) for i in range(1, n))


def count_plans(n, n_mp):
    """All (contiguous partition, per-block MP) pairs: Eq. 4 plus its missing i = 0 term
    (the single block), which sums to n_mp * (1 + n_mp)^(n-1)."""
    return n_mp * (1 + n_mp) ** (n - 1)


def enumerate_partitions(n):
    """Every way to cut layers 0..n-1 into contiguous blocks, as tuples of last indices."""
    for cuts in itertools.product((0, 1), repeat=n - 1):
        yield tuple([i for i in range(n - 1) if cuts[i]] + [n - 1])


def enumerate_plans(n, budgets):
    """Every (group_last tuple, budget tuple) pair."""
    for part in enumerate_partitions(n):
        for b in itertools.product(budgets, repeat=len(part)):
            yield part, b


def best_plan_exhaustive(n, budgets, cost_fn):
    """Brute force over enumerate_plans.  cost_fn(first, last, budget) -> int cost, or None if the
    block cannot be executed.  The winner is the minimum under the total order
    (total cost, number of blocks, group_last lexicographic, budgets lexicographic).
    Returns (cost, group_last, budgets, number_of_plans_visited)."""
    table = {}
    for f in range(n):
        for l in range(f, n):
            for b in budgets:
                table[(f, l, b)] = cost_fn(f, l, b)
    best = None
    visited = 0
    for part, bud in enumerate_plans(n, budgets):
        visited += 1
        total = 0
        first = 0
        ok = True
        for last, b in zip(part, bud):
            c = table[(first, last, b)]
            if c is None:
                ok = False
                break
            total += c
            first = last + 1
        if not ok:
            continue
        key = (total, len(part), part, bud)
        if best is None or key < best:
            best = key
    if best is None:
        return None, None, None, visited
    return best[0], best[2], best[3], visited


# --------------------------------------------------------------------------------------------
# Per-layer MP (Eq. 5) and the greedy joint pass (Algorithm 1)
# --------------------------------------------------------------------------------------------

def layer_mp(L, ops, alpha, beta, k, b, max_mp):
    """Eq. 5 gives MP only up to proportionality: MP ~ alpha*log2(C) + beta*log2(OpCount).
    Reading used here: C = min(Cin, Cout); MP = k*score + b with hardware-fitted k, b; clamped
    to [1, max_mp]; kept real-valued (rounding happens once per block)."""
    c = min(L["cin"], L["cout"])
    score = alpha * math.log2(c) + beta * math.log2(ops)
    return min(float(max_mp), max(1.0, k * score + b))


def round_block_mp(avg_mp, allowed):
    """Block MP = 2^floor(log2(avg)), then the largest allowed value not above it (the smallest
    allowed value if none is)."""
    p = 2 ** int(math.floor(math.log2(avg_mp)))
    below = [a for a in allowed if a <= p]
    return max(below) if below else min(allowed)


def algorithm1(layers, ops, opcount_critical, alpha=0.316, beta=0.659, k=1.0, b=0.0,
               allowed=(1, 2, 4, 8, 16, 32)):
    """Greedy O(n) pass of Algorithm 1 ("Finding fusion scheme and hyper-parameter setting").

    layers: layer dicts; ops[i]: operation count of layer i (Eq. 1/2).  Walk the layers once; a
    convolution or FC layer contributes its Eq.-5 MP and its operation count to the open block;
    after every layer the block's average MP is recomputed and the block is closed as soon as
    (summed operations / average MP) reaches opcount_critical; its MP is the rounded average.

    Readings where the printed listing is silent or inconsistent: the running mean is kept as a
    sum and a count (not overwritten by the division); the threshold test is skipped while the
    block holds no conv/FC layer; the loop covers 0 <= i < n; layers left over when the loop ends
    form a last block; trailing pool layers after a closing layer ride with that block (a block
    never starts with a pooling layer).
    Returns (fusion_partition_index, mp_of_fusionblock).
    """
    n = len(layers)
    max_mp = max(allowed)
    part, mps = [], []
    sum_op, sum_mp, block_size = 0, 0.0, 0
    i = 0
    while i < n:
        L = layers[i]
        if L["op"] in CONV_LIKE:
            sum_mp += layer_mp(L, ops[i], alpha, beta, k, b, max_mp)
            sum_op += ops[i]
            block_size += 1
        if block_size > 0:
            avg = sum_mp / block_size
            if sum_op / avg >= opcount_critical:
                while i + 1 < n and layers[i + 1]["op"] not in CONV_LIKE:
                    i += 1
                part.append(i)
                mps.append(round_block_mp(avg, allowed))
                sum_op, sum_mp, block_size = 0, 0.0, 0
        i += 1
    covered = part[-1] + 1 if part else 0
    if covered < n:
        if block_size > 0:
            part.append(n - 1)
            mps.append(round_block_mp(sum_mp / block_size, allowed))
        elif part:
            part[-1] = n - 1
        else:
            part.append(n - 1)
            mps.append(min(allowed))
    return part, mps


def layerwise_budgets(layers, ops, alpha=0.316, beta=0.659, k=1.0, b=0.0, allowed=(1, 2, 4, 8, 16, 32),
                      fixed_budget=0):
    """The no-fusion strategies of the evaluation (Sec. V, table of strategies): every layer is a
    block of its own.  Strategy 3 gives each convolution / FC layer the MP of Eq. 5 (rounded as a
    block of one layer would be); strategies 1 and 2 use one MP for all (fixed_budget).  A layer
    without Eq.-5 features (pooling) takes the MP of the convolution before it (the smallest
    allowed MP if there is none).  Returns the per-layer MP list."""
    out = []
    cur = min(allowed)
    for i, L in enumerate(layers):
        if L["op"] in CONV_LIKE:
            cur = round_block_mp(layer_mp(L, ops[i], alpha, beta, k, b, max(allowed)), allowed)
        out.append(fixed_budget if fixed_budget > 0 else cur)
    return out


def max_fusion(n, feasible, budget):
    """Strategy 4 ("all fusion, maximal MP") as far as the kernels allow: walking left to right,
    each block is the longest range [first, last] that can run as one group (feasible(first, last)
    is the caller's test), all on the same MP.  Returns [(first, last, budget), ...]."""
    out = []
    first = 0
    while first < n:
        last = n - 1
        while not feasible(first, last):
            last -= 1
            assert last >= first, "a single layer must be feasible"
        out.append((first, last, budget))
        first = last + 1
    return out

