"""TEST INFRASTRUCTURE -- not part of the product.

Oracle for the choice of the resident experts of one MoE layer (eMoE Section 3.4,
Eq. 2, and the last paragraph of Section 3.2.2).  Plain Python loops and fp64, in
the paper's order and notation; nothing here is shared with the HIP library.

Steps:
  W1  observed workload: how many tokens each expert receives under ordinary
      (unrestricted) top-k routing -- Section 3.2.2: workload = "the total number
      of tokens" an expert receives.
  W2  expected tokens per expert, Eq. 2, per task type:
          N_i = (sum_{j<T} W_j + T * W_o) * s * f_i
      and the total over task types (Section 3.4).
  W3  the L experts with the largest totals, in descending order (Section 3.4).
  W4  the load list: selected experts that are not resident go into slots, the
      ones with the higher workload first; experts that were not selected leave
      the GPU (Section 3.2.2).

Readings where the paper is silent:
  * ties in W3: the lower expert index ranks first;
  * W4 slot choice: a new expert takes the lowest-numbered slot that is empty or
    holds an expert that was not selected; selected experts that are already
    resident stay where they are; after the new experts are placed, every other
    slot that still holds an unselected expert is emptied (ascending slot order).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def observed_workload(topk_unrestricted: np.ndarray, E: int) -> np.ndarray:
    """W1.  `topk_unrestricted[T, k]`: the experts each token would use with all experts present."""
    counts = [0] * E
    for row in np.asarray(topk_unrestricted):
        for e in row:
            counts[int(e)] += 1
    return np.asarray(counts, dtype=np.int64)


def expected_tokens(freq: np.ndarray, request_task: Sequence[int], request_tokens: Sequence[int],
                    w_out: Sequence[float], sensitive: Sequence[int]) -> np.ndarray:
    """W2.  freq[n_tasks, E] = f_i per task type; request j belongs to task request_task[j] and
    has request_tokens[j] = W_j input tokens; w_out[task] = W_o; sensitive[task] = s."""
    freq = np.asarray(freq, dtype=np.float64)
    n_tasks, E = freq.shape
    total = [0.0] * E
    for task in range(n_tasks):
        T = 0
        sum_w = 0.0
        for j, tk in enumerate(request_task):
            if int(tk) == task:
                T += 1
                sum_w += float(request_tokens[j])
        load = sum_w + T * float(w_out[task])
        s = 1.0 if int(sensitive[task]) else 0.0
        for i in range(E):
            total[i] += load * s * float(freq[task, i])
    return np.asarray(total, dtype=np.float64)


def select_top(expected: np.ndarray, L: int) -> np.ndarray:
    """W3.  Indices of the L largest entries, descending; equal entries in ascending index order."""
    order = sorted(range(len(expected)), key=lambda i: (-float(expected[i]), i))
    return np.asarray(order[:L], dtype=np.int32)


def plan_load(expert_of_slot: Sequence[int], selected: Sequence[int]) -> Tuple[List[int], List[int], np.ndarray]:
    """W4.  Returns (expert_ids, slot_ids, expert_of_slot afterwards); expert id -1 = empty the slot.
    `selected` is in descending workload order; raises if the slots cannot hold it."""
    eos = [int(e) for e in expert_of_slot]
    chosen = [int(e) for e in selected]
    if len(chosen) > len(eos):
        raise ValueError("more selected experts than slots")
    keep = set(chosen)
    experts: List[int] = []
    slots: List[int] = []
    for e in chosen:  # higher workload first
        if e in eos:
            continue
        s = next(i for i, cur in enumerate(eos) if cur < 0 or cur not in keep)
        eos[s] = e
        experts.append(e)
        slots.append(s)
    for s, cur in enumerate(eos):
        if cur >= 0 and cur not in keep:
            eos[s] = -1
            experts.append(-1)
            slots.append(s)
    return experts, slots, np.asarray(eos, dtype=np.int32)


REUSE, LOAD_ALL, PREDICT = 0, 1, 2


def prompt_action(index: int, period: int, all_experts_fit: bool = True) -> int:
    """Section 3.3: requests are numbered 0, 1, 2, ...; the first loads every expert; every p-th one
    invokes the predictor and loads what it predicts; the others reuse what is loaded.
    Reading where the paper is silent: if the slots cannot hold all experts, the first request
    needs a prediction too."""
    if index == 0:
        return LOAD_ALL if all_experts_fit else PREDICT
    return PREDICT if index % period == 0 else REUSE
