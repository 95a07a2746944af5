"""TEST INFRASTRUCTURE -- not part of the product.

Python face of the fp64 CPU oracle in `emoe_oracle.c` (built with gcc on first
use, or by `build_oracle()`).  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the HIP library and its binding never
do, and this package imports nothing from them.

Step names follow the layer's definition in `emoe_oracle.c`:
O1 gate logits, O2 restricted top-k, O3 gate weights, O4 permutation,
O5 expert FFN, O6 weighted combine.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "emoe_oracle.c")
_LIB = os.path.join(_HERE, "libemoe_oracle.so")

F32, BF16 = 0, 1
SWIGLU, RELU = 0, 1
ERR_RESIDENT = -4
_DTYPE = {"f32": F32, "bf16": BF16}
_ACT = {"swiglu": SWIGLU, "relu": RELU}


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"oracle {where} failed with code {code}")
        self.code = code


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle into a shared library next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _c():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build_oracle())
        for name in ("oracle_gate_logits", "oracle_route_mask_then_topk", "oracle_route_rank_then_skip",
                     "oracle_route_unrestricted", "oracle_permute", "oracle_gather_rows",
                     "oracle_expert_ffn_rows", "oracle_combine_tokens", "oracle_num_threads", "oracle_set_num_threads"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _check(rc: int, where: str):
    if rc != 0:
        raise OracleError(rc, where)


def num_threads() -> int:
    return int(_c().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads for the loops over independent rows (for timing the oracle as a baseline; results do not depend on it)."""
    _c().oracle_set_num_threads(int(n))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


# ---------------------------------------------------------------- O1
def gate_logits(x: np.ndarray, w_gate: np.ndarray, gate_bias: Optional[np.ndarray], dtype: str) -> np.ndarray:
    T, d = x.shape
    E = w_gate.shape[0]
    assert w_gate.shape[1] == d
    logits = np.empty((T, E), dtype=np.float64)
    b = None if gate_bias is None else np.ascontiguousarray(gate_bias, dtype=np.float32)
    _check(_c().oracle_gate_logits(T, d, E, _DTYPE[dtype], _p(x), _p(w_gate), _p(b), _p(logits)), "gate_logits")
    return logits


# ---------------------------------------------------------------- O2 + O3
def route(logits: np.ndarray, slot_of_expert: np.ndarray, k: int, formulation: str = "mask_then_topk"):
    """Returns (topk_expert [T,k] int32, topk_weight [T,k] float64)."""
    T, E = logits.shape
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    soe = _i32(slot_of_expert)
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float64)
    fn = {"mask_then_topk": _c().oracle_route_mask_then_topk,
          "rank_then_skip": _c().oracle_route_rank_then_skip}[formulation]
    _check(fn(T, E, k, _p(logits), _p(soe), _p(idx), _p(w)), "route/" + formulation)
    return idx, w


def route_unrestricted(logits: np.ndarray, k: int) -> np.ndarray:
    T, E = logits.shape
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    idx = np.empty((T, k), dtype=np.int32)
    _check(_c().oracle_route_unrestricted(T, E, k, _p(logits), _p(idx)), "route_unrestricted")
    return idx


# ---------------------------------------------------------------- O4
@dataclass
class Permutation:
    slot_counts: np.ndarray   # [S] int32
    slot_offsets: np.ndarray  # [S+1] int32
    perm: np.ndarray          # [A] int32: row r holds assignment perm[r]
    inv_perm: np.ndarray      # [A] int32: assignment a sits in row inv_perm[a]


def permute(topk_expert: np.ndarray, slot_of_expert: np.ndarray, S: int) -> Permutation:
    T, k = topk_expert.shape
    idx = _i32(topk_expert)
    soe = _i32(slot_of_expert)
    A = T * k
    counts = np.empty(S, dtype=np.int32)
    offsets = np.empty(S + 1, dtype=np.int32)
    perm = np.empty(A, dtype=np.int32)
    inv = np.empty(A, dtype=np.int32)
    _check(_c().oracle_permute(T, k, soe.shape[0], S, _p(idx), _p(soe), _p(counts), _p(offsets), _p(perm), _p(inv)),
           "permute")
    return Permutation(counts, offsets, perm, inv)


def gather_rows(x: np.ndarray, perm: np.ndarray, k: int, dtype: str) -> np.ndarray:
    A = perm.shape[0]
    d = x.shape[1]
    out = np.empty((A, d), dtype=x.dtype)
    _check(_c().oracle_gather_rows(A, k, d, _DTYPE[dtype], _p(x), _p(_i32(perm)), _p(out)), "gather_rows")
    return out


# ---------------------------------------------------------------- O5
def expert_ffn_rows(row_token: Sequence[int], row_slot: Sequence[int], x: np.ndarray, w1_slots: np.ndarray,
                    w3_slots: Optional[np.ndarray], w2_slots: np.ndarray, act: str, dtype: str,
                    return_h: bool = False):
    """y[n,:] for row n = FFN of slot row_slot[n] applied to token row_token[n]."""
    rt, rs = _i32(row_token), _i32(row_slot)
    n = rt.shape[0]
    S, f, d = w1_slots.shape
    assert w2_slots.shape == (S, d, f) and x.shape[1] == d
    assert n == 0 or (rs.min() >= 0 and rs.max() < S and rt.min() >= 0 and rt.max() < x.shape[0])
    y = np.empty((n, d), dtype=np.float64)
    h = np.empty((n, f), dtype=np.float64) if return_h else None
    _check(_c().oracle_expert_ffn_rows(n, _p(rt), _p(rs), d, f, _ACT[act], _DTYPE[dtype], _p(x), _p(w1_slots),
                                       _p(w3_slots), _p(w2_slots), _p(y), _p(h)), "expert_ffn_rows")
    return (y, h) if return_h else y


# ---------------------------------------------------------------- O6
def combine_tokens(tokens: Sequence[int], topk_weight: np.ndarray, row_index: np.ndarray,
                   y_rows: np.ndarray) -> np.ndarray:
    """out[n,:] = sum_j w[tokens[n], j] * y_rows[row_index[n, j], :]."""
    tk = _i32(tokens)
    k = topk_weight.shape[1]
    d = y_rows.shape[1]
    w = np.ascontiguousarray(topk_weight, dtype=np.float64)
    ri = _i32(row_index)
    yr = np.ascontiguousarray(y_rows, dtype=np.float64)
    out = np.empty((tk.shape[0], d), dtype=np.float64)
    _check(_c().oracle_combine_tokens(tk.shape[0], _p(tk), k, d, _p(w), _p(ri), _p(yr), _p(out)), "combine")
    return out


# ---------------------------------------------------------------- whole layer
@dataclass
class LayerResult:
    logits: np.ndarray
    topk_expert: np.ndarray
    topk_weight: np.ndarray
    permutation: Permutation
    tokens: np.ndarray                  # tokens for which `out` was computed
    out: Optional[np.ndarray]           # [len(tokens), d] float64
    y_rows: Dict[int, np.ndarray]       # permuted row index -> y row (float64), for the rows computed
    h_rows: Optional[Dict[int, np.ndarray]] = None   # the same rows of the intermediate h (float64)


def layer_forward(inp, tokens: Optional[Sequence[int]] = None, with_ffn: bool = True) -> LayerResult:
    """O1..O6 on a `LayerInputs`-shaped object (fields x, w_gate, gate_bias, slot_of_expert,
    w1_slots, w3_slots, w2_slots, cfg).  `tokens` restricts O5/O6 to a sample of tokens;
    routing and the permutation are always computed for all T tokens."""
    cfg = inp.cfg
    T, k, S = cfg.T, cfg.k, cfg.slots
    logits = gate_logits(inp.x, inp.w_gate, inp.gate_bias, cfg.dtype)
    idx, w = route(logits, inp.slot_of_expert, k, "mask_then_topk")
    idx_b, w_b = route(logits, inp.slot_of_expert, k, "rank_then_skip")
    if not (np.array_equal(idx, idx_b) and np.array_equal(w, w_b)):
        raise OracleError(-100, "the two formulations of restricted top-k disagree")
    pm = permute(idx, inp.slot_of_expert, S)
    tok = np.arange(T, dtype=np.int32) if tokens is None else _i32(tokens)
    if not with_ffn:
        return LayerResult(logits, idx, w, pm, tok, None, {})
    # rows needed: for token t and choice j, row r = inv_perm[t*k + j]; its slot is that of expert idx[t,j]
    a = (tok[:, None].astype(np.int64) * k + np.arange(k)[None, :]).reshape(-1)
    rows = pm.inv_perm[a]
    row_token = (pm.perm[rows] // k).astype(np.int32)
    row_slot = np.asarray(inp.slot_of_expert)[idx.reshape(-1)[a]].astype(np.int32)
    y, h = expert_ffn_rows(row_token, row_slot, inp.x, inp.w1_slots, inp.w3_slots, inp.w2_slots, cfg.act, cfg.dtype,
                           return_h=True)
    row_index = np.arange(a.shape[0], dtype=np.int32).reshape(-1, k)
    out = combine_tokens(tok, w, row_index, y)
    return LayerResult(logits, idx, w, pm, tok, out, {int(r): y[i] for i, r in enumerate(rows)},
                       {int(r): h[i] for i, r in enumerate(rows)})
