"""Seeded synthetic inputs for the resident-expert MoE layer.

This module only draws random numbers, rounds them to the storage type and
lays them out in memory.  It serves both the CPU oracle and the HIP path and
therefore contains none of the layer's arithmetic that either side is graded
on: it never produces an expected value.  The one computation it performs on
its own draws is an input *filter* (`_rows_below_margin`): token rows whose
resident gate logits are closer together than a margin are redrawn, so that
routing decisions are insensitive to the accumulation precision of whoever
consumes the inputs.  The filter's numbers are discarded afterwards.

The shapes follow the models the paper serves (Section 2.1: Mixtral-8x7B,
OpenMoE, top-1/top-2 gates); the structure follows what the paper reports about
its workloads: a few popular experts (Section 1) -> Zipf-distributed gate bias,
and only a fraction of experts resident on the GPU (Sections 3.2.2, 5.5).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 2503068230
MARGIN = 1e-2

F32 = "f32"
BF16 = "bf16"
SWIGLU = "swiglu"
RELU = "relu"


@dataclass(frozen=True)
class LayerConfig:
    """Shape of one MoE layer plus the recipe for its resident set.

    T tokens, d_model, d_ff, E experts, k experts per token, R resident
    experts, S slots (S >= R).  `zipf_s` > 0 adds a gate bias
    b[e] = -zipf_s * ln(rank_e) with a seeded rank permutation.  `resident`
    is "seeded" (uniform subset) or "popular" (the R best-ranked experts).
    """
    name: str
    index: int
    T: int
    d_model: int
    d_ff: int
    E: int
    k: int
    R: int
    dtype: str
    act: str
    zipf_s: float = 0.0
    resident: str = "seeded"
    S: int = 0  # 0 -> S = R

    @property
    def slots(self) -> int:
        return self.S if self.S > 0 else self.R

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def n_mats(self) -> int:
        return 3 if self.act == SWIGLU else 2

    @property
    def params_per_expert(self) -> int:
        return self.n_mats * self.d_model * self.d_ff

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


C1 = LayerConfig("C1_tiny_f32", 0, 64, 128, 256, 8, 2, 4, F32, SWIGLU)
C2 = LayerConfig("C2_switch_bf16", 1, 1024, 768, 3072, 64, 1, 16, BF16, RELU, zipf_s=1.1)
C3 = LayerConfig("C3_mixtral_prefill_bf16", 2, 4096, 4096, 14336, 8, 2, 4, BF16, SWIGLU)
C4 = LayerConfig("C4_mixtral_decode_bf16", 3, 64, 4096, 14336, 8, 2, 6, BF16, SWIGLU)
C5 = LayerConfig("C5_finegrained_bf16", 4, 8192, 2048, 1408, 64, 6, 24, BF16, SWIGLU,
                 zipf_s=1.2, resident="popular")
CONFIGS = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5}
# Further shapes of the model families the paper serves (Section 2.1), not part of the graded five:
# a Mixtral-8x22B-shaped prefill layer, an OpenMoE-shaped layer (32 experts, top-2, half resident)
X1 = LayerConfig("X1_mixtral_8x22b_prefill_bf16", 5, 4096, 6144, 16384, 8, 2, 4, BF16, SWIGLU)
X2 = LayerConfig("X2_openmoe_like_bf16", 6, 2048, 2048, 8192, 32, 2, 16, BF16, SWIGLU, zipf_s=1.1)
# one short prompt at the Mixtral-8x7B shape (a few dozen rows per expert: between a decode step and a batch of prompts)
X3 = LayerConfig("X3_mixtral_one_prompt_bf16", 7, 256, 4096, 14336, 8, 2, 6, BF16, SWIGLU)
# two prompts of 512 tokens with every expert resident (the first prompt of Section 3.3): about 256 rows per slot
X4 = LayerConfig("X4_mixtral_two_prompts_bf16", 8, 1024, 4096, 14336, 8, 2, 8, BF16, SWIGLU)
# a decode step of 128 tokens with every expert resident: 32 rows per slot on average, between the streaming
# kernels' range and a prompt's
X5 = LayerConfig("X5_mixtral_decode128_bf16", 9, 128, 4096, 14336, 8, 2, 8, BF16, SWIGLU)
EXTRA_CONFIGS = {"X1": X1, "X2": X2, "X3": X3, "X4": X4, "X5": X5}


def small_variant(cfg: LayerConfig, *, T: Optional[int] = None, d_model: Optional[int] = None,
                  d_ff: Optional[int] = None, name: Optional[str] = None) -> LayerConfig:
    """Same structure as `cfg` with smaller extents (for oracle-sized parity cases)."""
    return replace(cfg, T=T or cfg.T, d_model=d_model or cfg.d_model, d_ff=d_ff or cfg.d_ff,
                   name=name or (cfg.name + "_small"))


# --------------------------------------------------------------------------
# storage-type helpers (format conversion only)
# --------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values -> array in the layer's storage type (float32, or uint16 bf16 bits)."""
    if dtype == F32:
        return np.ascontiguousarray(a, dtype=np.float32)
    return f32_to_bf16_bits(a)


def storage_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage array to float64."""
    if dtype == F32:
        return a.astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


# --------------------------------------------------------------------------
# the generator
# --------------------------------------------------------------------------

def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


# stream ids under one config seed
_STREAM_X, _STREAM_WG, _STREAM_RANK, _STREAM_RESIDENT, _STREAM_SLOTS, _STREAM_REDRAW = range(6)
_STREAM_EXPERT = 1000


def expert_weights(cfg: LayerConfig, e: int, seed: Optional[int] = None
                   ) -> Tuple[np.ndarray, Optional[np.ndarray], np.ndarray]:
    """Weights of expert `e` in canonical layout and storage type.

    W1 [d_ff, d_model], W3 [d_ff, d_model] (None for ReLU), W2 [d_model, d_ff];
    W1, W3 ~ N(0, std = 1/sqrt(d_model)), W2 ~ N(0, std = 1/sqrt(d_ff)).
    Each expert has its own random stream, so an expert's weights do not depend
    on which other experts are generated.
    """
    seed = cfg.seed if seed is None else seed
    g = _rng(seed, _STREAM_EXPERT + e)
    d, f = cfg.d_model, cfg.d_ff
    s_in = np.float32(1.0 / np.sqrt(d))
    s_ff = np.float32(1.0 / np.sqrt(f))
    w1 = to_storage(g.standard_normal((f, d), dtype=np.float32) * s_in, cfg.dtype)
    w3 = None
    if cfg.act == SWIGLU:
        w3 = to_storage(g.standard_normal((f, d), dtype=np.float32) * s_in, cfg.dtype)
    w2 = to_storage(g.standard_normal((d, f), dtype=np.float32) * s_ff, cfg.dtype)
    return w1, w3, w2


def _rows_below_margin(x_rows: np.ndarray, w_gate64: np.ndarray, bias: Optional[np.ndarray],
                       resident: np.ndarray, k: int, dtype: str) -> np.ndarray:
    """Input filter: which rows have two of their top-(k+1) resident gate logits closer than MARGIN.

    Used only to decide which rows to redraw; nothing computed here is handed on.
    """
    lg = storage_to_f64(x_rows, dtype) @ w_gate64.T
    if bias is not None:
        lg = lg + bias.astype(np.float64)[None, :]
    lg = lg[:, resident]
    n_top = min(k + 1, lg.shape[1])
    top = -np.sort(-lg, axis=1)[:, :n_top]
    gaps = top[:, :-1] - top[:, 1:]
    if gaps.shape[1] == 0:
        return np.zeros(lg.shape[0], dtype=bool)
    return gaps.min(axis=1) < MARGIN


@dataclass
class LayerInputs:
    cfg: LayerConfig
    seed: int
    x: np.ndarray                    # [T, d] storage
    w_gate: np.ndarray               # [E, d] storage
    gate_bias: Optional[np.ndarray]  # [E] float32 or None
    slot_of_expert: np.ndarray       # [E] int32, -1 = not resident
    expert_of_slot: np.ndarray       # [S] int32, -1 = empty slot
    w1_slots: Optional[np.ndarray] = None  # [S, f, d] storage
    w3_slots: Optional[np.ndarray] = None  # [S, f, d] storage (None for ReLU)
    w2_slots: Optional[np.ndarray] = None  # [S, d, f] storage
    meta: Dict[str, object] = field(default_factory=dict)

    @property
    def resident_experts(self) -> np.ndarray:
        return np.flatnonzero(self.slot_of_expert >= 0).astype(np.int32)


def make_routing_inputs(cfg: LayerConfig, seed: Optional[int] = None, *, shuffle_slots: bool = False,
                        resident_override: Optional[np.ndarray] = None,
                        enforce_margin: bool = True) -> LayerInputs:
    """x, gate weights, gate bias and the resident set / slot map (no expert weights)."""
    seed = cfg.seed if seed is None else seed
    T, d, E, k, R, S = cfg.T, cfg.d_model, cfg.E, cfg.k, cfg.R, cfg.slots
    assert 1 <= k <= R <= S <= E, "need 1 <= k <= R <= S <= E"

    x = to_storage(_rng(seed, _STREAM_X).standard_normal((T, d), dtype=np.float32), cfg.dtype)
    w_gate = to_storage(_rng(seed, _STREAM_WG).standard_normal((E, d), dtype=np.float32)
                        * np.float32(1.0 / np.sqrt(d)), cfg.dtype)

    rank = _rng(seed, _STREAM_RANK).permutation(E) + 1          # rank[e] in 1..E
    gate_bias = None
    if cfg.zipf_s > 0:
        gate_bias = (-cfg.zipf_s * np.log(rank.astype(np.float64))).astype(np.float32)

    if resident_override is not None:
        resident = np.sort(np.asarray(resident_override, dtype=np.int64))
        assert len(resident) == R
    elif cfg.resident == "popular":
        resident = np.sort(np.argsort(rank, kind="stable")[:R])
    else:
        resident = np.sort(_rng(seed, _STREAM_RESIDENT).choice(E, size=R, replace=False))

    slots = np.arange(R)
    if shuffle_slots:
        slots = _rng(seed, _STREAM_SLOTS).permutation(S)[:R]
    slot_of_expert = np.full(E, -1, dtype=np.int32)
    expert_of_slot = np.full(S, -1, dtype=np.int32)
    slot_of_expert[resident] = slots
    expert_of_slot[slots] = resident

    redrawn = 0
    if enforce_margin and T > 0:
        wg64 = storage_to_f64(w_gate, cfg.dtype)
        g = _rng(seed, _STREAM_REDRAW)
        bad = np.flatnonzero(_rows_below_margin(x, wg64, gate_bias, resident, k, cfg.dtype))
        tries = 0
        while bad.size:
            tries += 1
            if tries > 100:
                raise RuntimeError("margin filter did not converge")
            x[bad] = to_storage(g.standard_normal((bad.size, d), dtype=np.float32), cfg.dtype)
            redrawn += int(bad.size)
            bad = bad[_rows_below_margin(x[bad], wg64, gate_bias, resident, k, cfg.dtype)]

    return LayerInputs(cfg=cfg, seed=seed, x=x, w_gate=w_gate, gate_bias=gate_bias,
                       slot_of_expert=slot_of_expert, expert_of_slot=expert_of_slot,
                       meta={"rows_redrawn": redrawn, "rank": rank})


def fill_slot_weights(inp: LayerInputs) -> LayerInputs:
    """Generate the resident experts' weights straight into slot-major buffers."""
    cfg = inp.cfg
    S, d, f = cfg.slots, cfg.d_model, cfg.d_ff
    np_dtype = np.float32 if cfg.dtype == F32 else np.uint16
    inp.w1_slots = np.zeros((S, f, d), dtype=np_dtype)
    inp.w2_slots = np.zeros((S, d, f), dtype=np_dtype)
    inp.w3_slots = np.zeros((S, f, d), dtype=np_dtype) if cfg.act == SWIGLU else None
    for s in range(S):
        e = int(inp.expert_of_slot[s])
        if e < 0:
            continue
        w1, w3, w2 = expert_weights(cfg, e, inp.seed)
        inp.w1_slots[s] = w1
        inp.w2_slots[s] = w2
        if w3 is not None:
            inp.w3_slots[s] = w3
    return inp


def make_layer_inputs(cfg: LayerConfig, seed: Optional[int] = None, **kw) -> LayerInputs:
    """Everything one layer forward needs: routing inputs plus resident slot weights."""
    return fill_slot_weights(make_routing_inputs(cfg, seed, **kw))
