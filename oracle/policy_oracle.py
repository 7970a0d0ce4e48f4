"""Plain definitions of the two CPU policies of the paper, written out step by step.

TEST INFRASTRUCTURE ONLY: the library's own implementations (heap-based, C++) are checked
against these; nothing of the product imports this file.

  arbitrate  — Sec. 5.2, Alg. 2 (GPU-local request scheduling): the Moore-Hodgson rule on
               prefill-completion deadlines d = a + s with execution times e = p / c.
  place      — Sec. 5.1, Alg. 1 (model placement to maximise memory headroom) with the
               tensor-parallel rule of the appendix "TP Support".

Readings where the paper is silent or garbled (the same as the library's header states):
equal deadlines / equal rates keep index order; among equally long requests the one earliest
in S is dropped; the update "r_k / s_k" of Alg. 1 means t_k * tz_k / s_k (its sort key); a GPU
with no memory left has infinite pressure; a model without a current GPU (-1) goes to the
best one; a tensor-parallel part goes to the lowest-pressure GPU that holds no sibling.
"""
import math


def arbitrate(arrival, slo, prompt_len, speed, now):
    """Sec. 5.2, Alg. 2.  The problem: one server, free from `now` on, jobs i with processing time
    cost_i = prompt_len_i / speed_i and due date due_i = arrival_i + slo_i; keep as many jobs as can
    all finish by their due dates when run back to back.  The Moore-Hodgson rule solves it: run
    through the jobs by rising due date, keep each, and whenever the kept jobs no longer all fit in
    front of the newcomer's due date, give up the costliest kept job.  Returns the kept indices in
    running order."""
    n = len(arrival)
    due = [arrival[i] + slo[i] for i in range(n)]
    cost = [prompt_len[i] / speed[i] for i in range(n)]
    kept = []                      # by rising due date
    busy_until = now               # when the kept jobs, run back to back, are done
    for i in sorted(range(n), key=lambda i: (due[i], i)):
        kept.append(i)
        busy_until = busy_until + cost[i]
        if busy_until > due[i]:
            victim = max(kept, key=lambda j: cost[j])      # the first of the costliest, in running order
            kept.remove(victim)
            busy_until = busy_until - cost[victim]
    return kept


def place(n_gpus, capacity, tau, token_rate, token_size, slo, weight, current_gpu=None, tp_group=None):
    """Sec. 5.1, Alg. 1 with the tensor-parallel rule of the appendix.  Every GPU is a pair (load, room):
    load = the summed SLO-weighted token rates of the models it hosts, room = capacity minus their
    weights; its KV pressure ratio is load / room (infinite once no room is left).  Models are dealt out
    by falling rate; each goes where the pressure is lowest, except that a model already living on a GPU
    whose pressure is at most tau above the lowest stays there (no migration for a small gain), and no
    two parts of one tensor-parallel model share a GPU."""
    n = len(token_rate)
    rate = [token_rate[j] * token_size[j] / slo[j] for j in range(n)]
    load, room = [0.0] * n_gpus, [capacity] * n_gpus
    home = [-1] * n

    def pressure(g):
        return load[g] / room[g] if room[g] > 0 else math.inf

    for j in sorted(range(n), key=lambda j: (-rate[j], j)):
        taken = set()                                        # GPUs that already host a sibling part
        if tp_group is not None and tp_group[j] >= 0:
            taken = {home[o] for o in range(n) if o != j and home[o] >= 0 and tp_group[o] == tp_group[j]}
        allowed = [g for g in range(n_gpus) if g not in taken]
        if not allowed:
            raise ValueError("more tensor-parallel parts than GPUs")
        calmest = min(allowed, key=lambda g: (pressure(g), g))
        here = -1 if current_gpu is None else current_gpu[j]
        stays = here >= 0 and here not in taken and not (pressure(here) - pressure(calmest) > tau)
        home[j] = here if stays else calmest
        load[home[j]] += rate[j]
        room[home[j]] -= weight[j]
    return home


def max_kvpr(n_gpus, capacity, placement, token_rate, token_size, slo, weight):
    """Largest KV pressure ratio over the GPUs of a finished placement."""
    rate = [0.0] * n_gpus
    shared = [capacity] * n_gpus
    for j, g in enumerate(placement):
        rate[g] += token_rate[j] * token_size[j] / slo[j]
        shared[g] -= weight[j]
    return max((rate[i] / shared[i]) if shared[i] > 0 else (math.inf if rate[i] > 0 or shared[i] < 0 else 0.0)
               for i in range(n_gpus))
