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
    n = len(arrival)
    R = sorted(range(n), key=lambda i: (arrival[i] + slo[i], i))          # ascending deadlines
    S = []
    current_time = now
    for r in R:
        e_r = prompt_len[r] / speed[r]
        S.append(r)
        current_time = current_time + e_r
        if current_time > arrival[r] + slo[r]:
            # pop the request with the longest execution time (the first such in S)
            longest = max(prompt_len[x] / speed[x] for x in S)
            r_max = next(x for x in S if prompt_len[x] / speed[x] == longest)
            S.remove(r_max)
            current_time = current_time - prompt_len[r_max] / speed[r_max]
    return S


def place(n_gpus, capacity, tau, token_rate, token_size, slo, weight, current_gpu=None, tp_group=None):
    M = len(token_rate)
    demand = [token_rate[j] * token_size[j] / slo[j] for j in range(M)]
    order = sorted(range(M), key=lambda j: (-demand[j], j))               # descending SLO-weighted rate
    shared_kv = [capacity] * n_gpus
    w_token_rate = [0.0] * n_gpus
    out = [-1] * M

    def kvpr(i):
        return w_token_rate[i] / shared_kv[i] if shared_kv[i] > 0 else math.inf

    for j in order:
        banned = set()
        if tp_group is not None and tp_group[j] >= 0:
            banned = {out[o] for o in range(M) if o != j and out[o] >= 0 and tp_group[o] == tp_group[j]}
        candidates = [i for i in range(n_gpus) if i not in banned]
        if not candidates:
            raise ValueError("more tensor-parallel parts than GPUs")
        best_idx = min(candidates, key=lambda i: (kvpr(i), i))
        best_r = kvpr(best_idx)
        g = -1 if current_gpu is None else current_gpu[j]
        if g >= 0 and g not in banned:
            current_r = kvpr(g)
            best_gpu = best_idx if current_r - best_r > tau else g
        else:
            best_gpu = best_idx
        out[j] = best_gpu
        w_token_rate[best_gpu] += demand[j]
        shared_kv[best_gpu] -= weight[j]
    return out


def max_kvpr(n_gpus, capacity, placement, token_rate, token_size, slo, weight):
    """Largest KV pressure ratio over the GPUs of a finished placement."""
    rate = [0.0] * n_gpus
    shared = [capacity] * n_gpus
    for j, g in enumerate(placement):
        rate[g] += token_rate[j] * token_size[j] / slo[j]
        shared[g] -= weight[j]
    return max((rate[i] / shared[i]) if shared[i] > 0 else (math.inf if rate[i] > 0 or shared[i] < 0 else 0.0)
               for i in range(n_gpus))
