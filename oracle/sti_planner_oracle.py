"""TEST INFRASTRUCTURE ONLY - slow reference of the two-stage planner.

Only tests/ may import this module; it shares no code with the library's planner.

What it computes (Section "Compute Planning", "IO Planning"):

* ``plan_submodel``: among all (n, m) with n layers of m shards whose computation fits the
  deadline, n * T_comp(m) <= T, the one with the most shards n*m; ties go to the deeper one.
* ``plan_bitwidths``: the two-pass allocation.  Validity is NOT checked through the paper's
  accumulated-IO-budget bookkeeping here but through the statement it encodes (Section
  "Accumulated IO Budgets", key idea): the pipeline does not stall iff, before a layer
  executes, all shards of this and of the earlier layers are loaded.  IO runs back to back
  in layer order and gets a head start equal to the time it took to fill the preload buffer;
  layer k starts at k * T_comp.  So a plan is valid iff for every layer k the IO time of all
  shards of layers 0..k (preloaded ones included, as the paper charges them) is at most the
  head start plus k * T_comp.
  Pass 1: the highest uniform bitwidth for all non-preloaded shards that keeps the plan
  valid (2 bits if none does, and then nothing more is allocated).  Pass 2: in order of
  decreasing importance, raise a non-preloaded shard to 32 bits whenever the plan stays valid.

Readings where the paper leaves a choice: the submodel is layers 0..n-1 x shards 0..m-1;
preloaded shards outside the submodel are ignored; preloaded shards keep their version;
the uniform bitwidth may be any of 2..6 or 32.
"""
from __future__ import annotations

BITWIDTHS = (2, 3, 4, 5, 6, 32)


def plan_submodel(t_comp, n_layers, deadline):
    """t_comp[m-1]: seconds per layer of m shards.  Returns (n, m), (0, 0) if nothing fits."""
    best = (0, 0)
    for n in range(1, n_layers + 1):
        for m in range(1, len(t_comp) + 1):
            if n * t_comp[m - 1] <= deadline:
                if (n * m, n) > (best[0] * best[1], best[0]):
                    best = (n, m)
    return best


def t_io_of(t_io, k):
    return t_io[BITWIDTHS.index(k)]


def stall_free(plan, preloaded, t_io, t_comp_m, n, m, M):
    """The timeline test described in the module docstring."""
    head_start = sum(t_io_of(t_io, preloaded[l * M + i]) for l in range(n) for i in range(m)
                     if preloaded[l * M + i])
    io_so_far = 0.0
    for k in range(n):
        io_so_far += sum(t_io_of(t_io, plan[k * M + i]) for i in range(m))
        if io_so_far > head_start + k * t_comp_m + 1e-12:
            return False
    return True


def plan_bitwidths(t_io, t_comp, N, M, n, m, preloaded, importance):
    """Returns (plan[N*M] of bitwidth-or-0, slack[n]) where slack[k] is the IO time still
    unused before layer k starts (the paper's AIB(k) after the allocation)."""
    plan = [0] * (N * M)
    if n == 0 or m == 0:
        return plan, []
    t_comp_m = t_comp[m - 1]
    free = []
    for l in range(n):
        for i in range(m):
            if preloaded[l * M + i]:
                plan[l * M + i] = preloaded[l * M + i]
            else:
                free.append(l * M + i)
    # pass 1
    chosen = None
    for k in BITWIDTHS:
        trial = list(plan)
        for s in free:
            trial[s] = k
        if stall_free(trial, preloaded, t_io, t_comp_m, n, m, M):
            chosen = k
    for s in free:
        plan[s] = chosen if chosen is not None else 2
    # pass 2
    if chosen is not None:
        for s in importance:
            l, i = divmod(s, M)
            if l >= n or i >= m or preloaded[s] or plan[s] == 32:
                continue
            trial = list(plan)
            trial[s] = 32
            if stall_free(trial, preloaded, t_io, t_comp_m, n, m, M):
                plan = trial
    head_start = sum(t_io_of(t_io, preloaded[l * M + i]) for l in range(n) for i in range(m)
                     if preloaded[l * M + i])
    slack, io_so_far = [], 0.0
    for k in range(n):
        io_so_far += sum(t_io_of(t_io, plan[k * M + i]) for i in range(m))
        slack.append(head_start + k * t_comp_m - io_so_far)
    return plan, slack
