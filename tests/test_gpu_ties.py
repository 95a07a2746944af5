"""GPU routing on inputs with exact ties (Section 3.2.2: the k best resident experts; the rule for equal
logits, lower expert index first, is this build's reading).  No margin filter here: token rows and
gate rows hold small integers, so every logit is an integer that fp32 accumulates exactly in any
order, and gate rows are repeated, so every token has experts with exactly equal logits: pairs of
two resident experts, of a resident and an absent one, inside and across the groups of experts that
one lane of the matrix-core kernel holds.  topk_expert and the observed workload must equal the
oracle's bit for bit, through both route kernels."""
import zlib

import numpy as np
import pytest
import torch

import emoe_inputs as gen
import oracle
import paper_2503_06823_amd as P
from gpu_util import TOL_WEIGHT, to_dev

pytestmark = pytest.mark.gpu

# (label, dtype, T, d_model, E, k, R, distinct gate rows, integer bias)
CASES = [
    ("f32_wave_per_token", "f32", 150, 96, 8, 2, 5, 3, False),
    ("f32_top1_bias", "f32", 90, 64, 16, 1, 6, 5, True),
    ("bf16_decode_wave_per_token", "bf16", 64, 2048, 12, 2, 7, 5, False),       # T <= 256, E <= 16, d >= 2048
    ("bf16_decode_wave_per_token_bias", "bf16", 200, 2048, 16, 3, 9, 6, True),
    ("bf16_mfma_E8", "bf16", 300, 256, 8, 2, 4, 3, False),
    ("bf16_mfma_E16_halves", "bf16", 700, 128, 16, 2, 9, 5, False),
    ("bf16_mfma_E32_all_lanes", "bf16", 1000, 192, 32, 4, 13, 7, True),
    ("bf16_mfma_E64_top6", "bf16", 1500, 256, 64, 6, 24, 11, True),
    ("bf16_mfma_E48_k_equals_R", "bf16", 260, 328, 48, 5, 5, 9, False),
    ("bf16_mfma_all_rows_equal", "bf16", 130, 128, 64, 3, 30, 1, False),         # every logit of a token equal
]


def tie_inputs(dtype, T, d, E, R, n_rows, with_bias, seed):
    rng = np.random.default_rng(seed)
    x = rng.integers(-3, 4, size=(T, d)).astype(np.float32)
    pool = rng.integers(-2, 3, size=(n_rows, d)).astype(np.float32)
    w_gate = pool[np.arange(E) % n_rows]                     # expert e repeats the row of e - n_rows, e - 2 n_rows, ...
    bias = None
    if with_bias:                                            # equal within a group of repeated rows, so the ties stay
        bias = rng.integers(-4, 5, size=n_rows).astype(np.float32)[np.arange(E) % n_rows]
    resident = np.sort(rng.choice(E, size=R, replace=False))
    soe = np.full(E, -1, dtype=np.int32)
    soe[resident] = rng.permutation(R).astype(np.int32)
    return gen.to_storage(x, dtype), gen.to_storage(w_gate, dtype), bias, soe


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0])
def test_equal_logits_go_to_the_lower_expert_index(gpu_device, case):
    label, dtype, T, d, E, k, R, n_rows, with_bias = case
    x, wg, bias, soe = tie_inputs(dtype, T, d, E, R, n_rows, with_bias, seed=zlib.crc32(label.encode()))
    logits = oracle.gate_logits(x, wg, bias, dtype)
    assert np.array_equal(logits, np.round(logits)) and np.abs(logits).max() < 2 ** 24      # exact in fp32
    idx, w = oracle.route(logits, soe, k, "mask_then_topk")
    idx_b, _ = oracle.route(logits, soe, k, "rank_then_skip")
    assert np.array_equal(idx, idx_b)
    # the inputs do hold ties where they matter: among the k + 1 best resident logits of most tokens
    res = logits[:, soe >= 0]
    top = -np.sort(-res, axis=1)[:, :min(k + 1, R)]
    tied = (top[:, :-1] == top[:, 1:]).any(axis=1) if top.shape[1] > 1 else np.zeros(T, bool)
    assert R == 1 or tied.mean() > 0.3, "the case holds too few ties to test anything"
    free = oracle.route_unrestricted(logits, k)
    workload = np.bincount(free.reshape(-1), minlength=E).astype(np.int64)

    desc = P.make_desc(T, d, 64, E, k, R, dtype, "swiglu")
    dx, dwg = to_dev(x, dtype), to_dev(wg, dtype)
    dbias = None if bias is None else torch.from_numpy(bias).cuda()
    dsoe = torch.from_numpy(soe).cuda()
    te = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
    tw = torch.zeros((T, k), dtype=torch.float32, device="cuda")
    P.emoe_route(desc, dx, dwg, dbias, dsoe, te, tw)
    torch.cuda.synchronize()
    assert np.array_equal(te.cpu().numpy(), idx), f"{label}: topk_expert differs on tied logits"
    assert np.abs(tw.cpu().numpy().astype(np.float64) - w).max() <= TOL_WEIGHT
    # the observing variant: same routing, and the workload under ordinary routing with the same tie rule
    te2 = torch.full_like(te, -7)
    counts = torch.zeros(E, dtype=torch.int64, device="cuda")
    P.emoe_route_observe(desc, dx, dwg, dbias, dsoe, te2, tw, counts)
    P.emoe_route_observe(desc, dx, dwg, dbias, dsoe, te2, tw, counts)       # counts accumulate
    torch.cuda.synchronize()
    assert np.array_equal(te2.cpu().numpy(), idx)
    assert np.array_equal(counts.cpu().numpy(), 2 * workload), f"{label}: observed workload differs on tied logits"
