"""ctypes binding of libemoe.so: argument marshalling only.

Every step of the layer runs in the HIP kernels behind the C ABI declared in include/emoe.h.
Tensor arguments are torch tensors (device memory comes from torch; `.data_ptr()` is what crosses
the boundary) or plain integer addresses.  There is no fallback: if the library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libemoe.so")

EMOE_OK = 0
EMOE_ERR_NULL, EMOE_ERR_SHAPE, EMOE_ERR_UNSUPPORTED = -1, -2, -3
EMOE_ERR_RESIDENT, EMOE_ERR_WORKSPACE, EMOE_ERR_DEVICE = -4, -5, -6
EMOE_F32, EMOE_BF16 = 0, 1
EMOE_ACT_SWIGLU, EMOE_ACT_RELU = 0, 1
DTYPES = {"f32": EMOE_F32, "bf16": EMOE_BF16}
ACTS = {"swiglu": EMOE_ACT_SWIGLU, "relu": EMOE_ACT_RELU}

EXPORTS = ("emoe_status_string", "emoe_workspace_bytes", "emoe_route", "emoe_route_observe", "emoe_permute",
           "emoe_permute_static",
           "emoe_expert_ffn", "emoe_expert_ffn_pass", "emoe_expert_ffn_gather", "emoe_expert_ffn_gather_pass", "emoe_expert_ffn_gather_combine", "emoe_combine",
           "emoe_layer_forward", "emoe_load_experts", "emoe_expected_tokens",
           "emoe_select_experts", "emoe_plan_load", "emoe_prompt_action", "emoe_loader_create", "emoe_loader_destroy",
           "emoe_loader_next_prompt", "emoe_loader_update", "emoe_loader_layer_begin", "emoe_loader_layer_end",
           "emoe_loader_layer_ready", "emoe_loader_residents", "emoe_loader_synchronize", "emoe_expected_latency", "emoe_schedule",
           "emoe_generation_tick", "emoe_measure_mfma_loop", "emoe_measure_read_stream",
           "emoe_measure_copy_stream", "emoe_measure_scatter_combine")


class EmoeLayerDesc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32),
                ("E", ctypes.c_int32), ("k", ctypes.c_int32), ("S", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("act", ctypes.c_int32)]


class EmoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {status_string(status)} (status {status})")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (see build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2503_06823_amd.build` "
                                    "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        dp = ctypes.POINTER(EmoeLayerDesc)
        L.emoe_status_string.restype = ctypes.c_char_p
        L.emoe_status_string.argtypes = [ctypes.c_int]
        L.emoe_workspace_bytes.argtypes = [dp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.emoe_route.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        L.emoe_permute.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.emoe_measure_mfma_loop.argtypes = [vp, sz, vp, sz, i32, i32, i32, vp, vp, vp]
        L.emoe_measure_read_stream.argtypes = [vp, sz, i32, vp, vp]
        L.emoe_measure_copy_stream.argtypes = [vp, vp, sz, i32, vp]
        L.emoe_measure_scatter_combine.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        L.emoe_permute_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.emoe_expert_ffn.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.emoe_expert_ffn_pass.argtypes = [dp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.emoe_combine.argtypes = [dp, vp, vp, vp, vp, vp]
        L.emoe_expert_ffn_gather_combine.argtypes = [dp] + [vp] * 11 + [sz, vp]
        L.emoe_layer_forward.argtypes = [dp] + [vp] * 15 + [vp, sz, vp, sz, vp]
        L.emoe_load_experts.argtypes = [dp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        for name in EXPORTS[1:]:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().emoe_status_string(int(status)).decode()


def make_desc(T: int, d_model: int, d_ff: int, E: int, k: int, S: int, dtype, act) -> EmoeLayerDesc:
    return EmoeLayerDesc(T, d_model, d_ff, E, k, S, DTYPES.get(dtype, dtype), ACTS.get(act, act))


def _ptr(t) -> ctypes.c_void_p:
    """Address of a torch tensor / numpy array / raw int / None."""
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if hasattr(t, "data_ptr"):
        return ctypes.c_void_p(t.data_ptr())
    if hasattr(t, "ctypes"):
        return ctypes.c_void_p(t.ctypes.data)
    raise TypeError(f"cannot take the address of {type(t)}")


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _event(ev) -> ctypes.c_void_p:
    if ev is None:
        return ctypes.c_void_p(0)
    if isinstance(ev, int):
        return ctypes.c_void_p(ev)
    handle = ev.cuda_event
    if not handle:
        # torch creates the HIP event at its first record(); before that there is no handle to pass, and
        # a NULL would silently mean "no event"
        raise ValueError("this torch event has no HIP event yet: create it with make_event(), or record it once")
    return ctypes.c_void_p(handle)


def make_event(timing: bool = False, stream=None):
    """A torch event whose HIP event exists (recorded once on `stream`, default the current one), so that
    it can be handed to the library as wait_event / done_event and be waited on or timed through torch."""
    import torch
    ev = torch.cuda.Event(enable_timing=timing)
    ev.record(stream if stream is not None else torch.cuda.current_stream())
    return ev


def _check(rc: int, where: str, check: bool) -> int:
    if check and rc != EMOE_OK:
        raise EmoeError(rc, where)
    return rc


def emoe_workspace_bytes(desc: EmoeLayerDesc, check: bool = True) -> Tuple[int, int]:
    a, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    rc = lib().emoe_workspace_bytes(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b))
    _check(rc, "emoe_workspace_bytes", check)
    return (a.value, b.value) if rc == EMOE_OK else (rc, rc)


def emoe_route(desc, x, w_gate, gate_bias, slot_of_expert, topk_expert, topk_weight, stream=None, check=True) -> int:
    rc = lib().emoe_route(ctypes.byref(desc), _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(slot_of_expert),
                          _ptr(topk_expert), _ptr(topk_weight), _stream(stream))
    return _check(rc, "emoe_route", check)


def emoe_route_observe(desc, x, w_gate, gate_bias, slot_of_expert, topk_expert, topk_weight, expert_tokens,
                       stream=None, check=True) -> int:
    """`expert_tokens`: int64 device tensor [E], accumulated."""
    rc = lib().emoe_route_observe(ctypes.byref(desc), _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(slot_of_expert),
                                  _ptr(topk_expert), _ptr(topk_weight), _ptr(expert_tokens), _stream(stream))
    return _check(rc, "emoe_route_observe", check)


def emoe_permute(desc, x, topk_expert, slot_of_expert, slot_counts, slot_offsets, perm, inv_perm, x_perm, ws,
                 ws_bytes, stream=None, check=True) -> int:
    rc = lib().emoe_permute(ctypes.byref(desc), _ptr(x), _ptr(topk_expert), _ptr(slot_of_expert), _ptr(slot_counts),
                            _ptr(slot_offsets), _ptr(perm), _ptr(inv_perm), _ptr(x_perm), _ptr(ws), int(ws_bytes),
                            _stream(stream))
    return _check(rc, "emoe_permute", check)


def emoe_permute_static(desc, x, topk_expert, slot_of_expert, slot_counts, slot_offsets, perm, inv_perm, x_perm,
                        stream=None, check=True) -> int:
    rc = lib().emoe_permute_static(ctypes.byref(desc), _ptr(x), _ptr(topk_expert), _ptr(slot_of_expert),
                                   _ptr(slot_counts), _ptr(slot_offsets), _ptr(perm), _ptr(inv_perm), _ptr(x_perm),
                                   _stream(stream))
    return _check(rc, "emoe_permute_static", check)


def emoe_measure_mfma_loop(a, b, lds_reads: bool, workgroups: int, iters: int, sink, stream=None) -> float:
    """Enqueues the matrix-instruction loop on the bf16 tensors a and b; returns the flop of the launch."""
    flop = ctypes.c_double(0.0)
    rc = lib().emoe_measure_mfma_loop(_ptr(a), ctypes.c_size_t(a.numel()), _ptr(b), ctypes.c_size_t(b.numel()),
                                      ctypes.c_int32(1 if lds_reads else 0), ctypes.c_int32(workgroups),
                                      ctypes.c_int32(iters), _ptr(sink), ctypes.byref(flop), _stream(stream))
    _check(rc, "emoe_measure_mfma_loop", True)
    return flop.value


def emoe_measure_read_stream(src, nbytes: int, workgroups: int, sink, stream=None) -> int:
    rc = lib().emoe_measure_read_stream(_ptr(src), ctypes.c_size_t(nbytes), ctypes.c_int32(workgroups), _ptr(sink),
                                        _stream(stream))
    return _check(rc, "emoe_measure_read_stream", True)


def emoe_measure_scatter_combine(desc, y_perm, perm, topk_weight, image, out, stream=None) -> int:
    rc = lib().emoe_measure_scatter_combine(ctypes.byref(desc), _ptr(y_perm), _ptr(perm), _ptr(topk_weight), _ptr(image),
                                            _ptr(out), _stream(stream))
    return _check(rc, "emoe_measure_scatter_combine", True)


def emoe_measure_copy_stream(src, dst, nbytes: int, workgroups: int, stream=None) -> int:
    rc = lib().emoe_measure_copy_stream(_ptr(src), _ptr(dst), ctypes.c_size_t(nbytes), ctypes.c_int32(workgroups),
                                        _stream(stream))
    return _check(rc, "emoe_measure_copy_stream", True)


def emoe_expert_ffn(desc, x_perm, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, ws_bytes, stream=None,
                    check=True) -> int:
    rc = lib().emoe_expert_ffn(ctypes.byref(desc), _ptr(x_perm), _ptr(slot_offsets), _ptr(w1_slots), _ptr(w3_slots),
                               _ptr(w2_slots), _ptr(y_perm), _ptr(ws), int(ws_bytes), _stream(stream))
    return _check(rc, "emoe_expert_ffn", check)


def emoe_expert_ffn_pass(desc, which, x_perm, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, ws_bytes,
                         stream=None, check=True) -> int:
    rc = lib().emoe_expert_ffn_pass(ctypes.byref(desc), int(which), _ptr(x_perm), _ptr(slot_offsets), _ptr(w1_slots),
                                    _ptr(w3_slots), _ptr(w2_slots), _ptr(y_perm), _ptr(ws), int(ws_bytes),
                                    _stream(stream))
    return _check(rc, "emoe_expert_ffn_pass", check)


def emoe_expert_ffn_gather(desc, x, perm, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, ws_bytes, stream=None,
                           check=True) -> int:
    rc = lib().emoe_expert_ffn_gather(ctypes.byref(desc), _ptr(x), _ptr(perm), _ptr(slot_offsets), _ptr(w1_slots),
                                      _ptr(w3_slots), _ptr(w2_slots), _ptr(y_perm), _ptr(ws),
                                      ctypes.c_size_t(int(ws_bytes)), _stream(stream))
    return _check(rc, "emoe_expert_ffn_gather", check)


def emoe_expert_ffn_gather_pass(desc, which, x, perm, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, ws_bytes,
                                stream=None, check=True) -> int:
    rc = lib().emoe_expert_ffn_gather_pass(ctypes.byref(desc), int(which), _ptr(x), _ptr(perm), _ptr(slot_offsets),
                                           _ptr(w1_slots), _ptr(w3_slots), _ptr(w2_slots), _ptr(y_perm), _ptr(ws),
                                           ctypes.c_size_t(int(ws_bytes)), _stream(stream))
    return _check(rc, "emoe_expert_ffn_gather_pass", check)


def emoe_expert_ffn_gather_combine(desc, x, perm, inv_perm, slot_offsets, w1_slots, w3_slots, w2_slots, topk_weight,
                                   y_perm, out, ws, ws_bytes, stream=None, check=True) -> int:
    rc = lib().emoe_expert_ffn_gather_combine(ctypes.byref(desc), _ptr(x), _ptr(perm), _ptr(inv_perm), _ptr(slot_offsets),
                                              _ptr(w1_slots), _ptr(w3_slots), _ptr(w2_slots), _ptr(topk_weight),
                                              _ptr(y_perm), _ptr(out), _ptr(ws), int(ws_bytes), _stream(stream))
    return _check(rc, "emoe_expert_ffn_gather_combine", check)


def emoe_combine(desc, y_perm, inv_perm, topk_weight, out, stream=None, check=True) -> int:
    rc = lib().emoe_combine(ctypes.byref(desc), _ptr(y_perm), _ptr(inv_perm), _ptr(topk_weight), _ptr(out),
                            _stream(stream))
    return _check(rc, "emoe_combine", check)


def emoe_layer_forward(desc, x, w_gate, gate_bias, slot_of_expert, w1_slots, w3_slots, w2_slots, topk_expert, topk_weight,
                       slot_counts, slot_offsets, perm, inv_perm, y_perm, out, permute_ws, permute_ws_bytes, ffn_ws,
                       ffn_ws_bytes, stream=None, check=True) -> int:
    rc = lib().emoe_layer_forward(ctypes.byref(desc), _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(slot_of_expert),
                                  _ptr(w1_slots), _ptr(w3_slots), _ptr(w2_slots), _ptr(topk_expert), _ptr(topk_weight),
                                  _ptr(slot_counts), _ptr(slot_offsets), _ptr(perm), _ptr(inv_perm), _ptr(y_perm),
                                  _ptr(out), _ptr(permute_ws), int(permute_ws_bytes), _ptr(ffn_ws), int(ffn_ws_bytes),
                                  _stream(stream))
    return _check(rc, "emoe_layer_forward", check)


def _i32_array(values: Optional[Sequence[int]]):
    if values is None:
        return None
    return (ctypes.c_int32 * len(values))(*[int(v) for v in values])


def _ptr_array(tensors: Optional[Sequence], E: int):
    """Host array of E host pointers (NULL where the caller gave None)."""
    if tensors is None:
        return None
    assert len(tensors) == E, "one entry (tensor or None) per expert"
    return (ctypes.c_void_p * E)(*[_ptr(t) for t in tensors])


def emoe_load_experts(desc, expert_ids, slot_ids, host_w1, host_w3, host_w2, w1_slots, w3_slots, w2_slots,
                      slot_of_expert, expert_of_slot, expert_of_slot_host, side_stream, wait_event=None,
                      done_event=None, check=True) -> int:
    """`host_w*`: sequences of E pinned host tensors (or None entries); `expert_of_slot_host`: a
    contiguous int32 numpy array or CPU tensor of length S, updated in place on success."""
    n = 0 if expert_ids is None else len(expert_ids)
    ids, slots = _i32_array(expert_ids), _i32_array(slot_ids)
    a1, a3, a2 = _ptr_array(host_w1, desc.E), _ptr_array(host_w3, desc.E), _ptr_array(host_w2, desc.E)
    cast = lambda a: ctypes.cast(a, ctypes.c_void_p) if a is not None else ctypes.c_void_p(0)
    rc = lib().emoe_load_experts(ctypes.byref(desc), n, cast(ids), cast(slots), cast(a1), cast(a3), cast(a2),
                                 _ptr(w1_slots), _ptr(w3_slots), _ptr(w2_slots), _ptr(slot_of_expert),
                                 _ptr(expert_of_slot), _ptr(expert_of_slot_host), _stream(side_stream),
                                 _event(wait_event), _event(done_event))
    return _check(rc, "emoe_load_experts", check)


def _host_array(ctype, values):
    values = list(values)
    return (ctype * max(len(values), 1))(*values), len(values)


def emoe_expected_tokens(freq, request_task, request_tokens, w_out, sensitive, check=True):
    """Eq. 2 on the host.  `freq`: n_tasks rows of E frequencies.  Returns the list of E totals (or the status)."""
    rows = [list(map(float, r)) for r in freq]
    n_tasks, E = len(rows), len(rows[0]) if rows else 0
    f, _ = _host_array(ctypes.c_double, [v for r in rows for v in r])
    rt, n_req = _host_array(ctypes.c_int32, [int(v) for v in request_task])
    rk, _ = _host_array(ctypes.c_int64, [int(v) for v in request_tokens])
    wo, _ = _host_array(ctypes.c_double, [float(v) for v in w_out])
    se, _ = _host_array(ctypes.c_int32, [int(v) for v in sensitive])
    out = (ctypes.c_double * max(E, 1))()
    rc = lib().emoe_expected_tokens(E, n_tasks, f, n_req, rt, rk, wo, se, out)
    _check(rc, "emoe_expected_tokens", check)
    return list(out)[:E] if rc == EMOE_OK else rc


def emoe_select_experts(expected, L, check=True):
    """The L experts with the largest expected token counts, descending.  Returns a list (or the status)."""
    e, E = _host_array(ctypes.c_double, [float(v) for v in expected])
    out = (ctypes.c_int32 * max(int(L), 1))()
    rc = lib().emoe_select_experts(E, e, int(L), out)
    _check(rc, "emoe_select_experts", check)
    return list(out)[:int(L)] if rc == EMOE_OK else rc


def emoe_plan_load(E, S, k, expert_of_slot_host, selected, check=True):
    """The (expert_ids, slot_ids) list for emoe_load_experts (or the status)."""
    eos, _ = _host_array(ctypes.c_int32, [int(v) for v in expert_of_slot_host])
    sel, L = _host_array(ctypes.c_int32, [int(v) for v in selected])
    ids, slots = (ctypes.c_int32 * max(int(S), 1))(), (ctypes.c_int32 * max(int(S), 1))()
    n = ctypes.c_int32(0)
    rc = lib().emoe_plan_load(int(E), int(S), int(k), eos, L, sel, ids, slots, ctypes.byref(n))
    _check(rc, "emoe_plan_load", check)
    return (list(ids)[:n.value], list(slots)[:n.value]) if rc == EMOE_OK else rc


EMOE_PROMPT_REUSE, EMOE_PROMPT_LOAD_ALL, EMOE_PROMPT_PREDICT = 0, 1, 2


def emoe_prompt_action(prompt_index: int, period: int, all_experts_fit: bool) -> int:
    return lib().emoe_prompt_action(ctypes.c_int64(int(prompt_index)), int(period), 1 if all_experts_fit else 0)


class EmoeLoaderLayer(ctypes.Structure):
    _fields_ = [("desc", EmoeLayerDesc),
                ("host_w1", ctypes.c_void_p), ("host_w3", ctypes.c_void_p), ("host_w2", ctypes.c_void_p),
                ("w1_slots", ctypes.c_void_p), ("w3_slots", ctypes.c_void_p), ("w2_slots", ctypes.c_void_p),
                ("slot_of_expert", ctypes.c_void_p), ("expert_of_slot", ctypes.c_void_p)]


class Loader:
    """Handle of an emoe_loader.  `layers`: one dict per MoE layer with keys desc, host_w1, host_w3, host_w2
    (sequences of E pinned host tensors), w1_slots, w3_slots, w2_slots, slot_of_expert, expert_of_slot (device
    tensors).  Keeps references to everything it handed to the library."""

    def __init__(self, layers, period: int):
        self._keep = []
        arr = (EmoeLoaderLayer * max(len(layers), 1))()
        for i, l in enumerate(layers):
            d = l["desc"]
            ptrs = [_ptr_array(l[k], d.E) for k in ("host_w1", "host_w3", "host_w2")]
            self._keep.append((l, ptrs))
            cast = lambda a: ctypes.cast(a, ctypes.c_void_p) if a is not None else None
            arr[i] = EmoeLoaderLayer(d, cast(ptrs[0]), cast(ptrs[1]), cast(ptrs[2]), _ptr(l["w1_slots"]),
                                     _ptr(l.get("w3_slots")), _ptr(l["w2_slots"]), _ptr(l["slot_of_expert"]),
                                     _ptr(l["expert_of_slot"]))
        self.n_layers = len(layers)
        self._slots = [l["desc"].S for l in layers]
        self._h = ctypes.c_void_p(0)
        rc = lib().emoe_loader_create(len(layers), arr, int(period), ctypes.byref(self._h))
        if rc != EMOE_OK:
            self._h = None
            raise EmoeError(rc, "emoe_loader_create")

    def next_prompt(self):
        """-> (prompt index, action)"""
        idx, act = ctypes.c_int64(0), ctypes.c_int32(0)
        _check(lib().emoe_loader_next_prompt(self._h, ctypes.byref(idx), ctypes.byref(act)), "emoe_loader_next_prompt", True)
        return idx.value, act.value

    def update(self, selected, check=True) -> int:
        """`selected`: per layer, the expert ids in descending workload order."""
        rows = [_i32_array(list(r)) for r in selected]
        ptrs = (ctypes.c_void_p * max(len(rows), 1))(*[ctypes.cast(r, ctypes.c_void_p) for r in rows])
        L = _i32_array([len(r) for r in selected])
        return _check(lib().emoe_loader_update(self._h, ptrs, L), "emoe_loader_update", check)

    def layer_begin(self, layer: int, stream=None) -> int:
        return _check(lib().emoe_loader_layer_begin(self._h, int(layer), _stream(stream)), "emoe_loader_layer_begin", True)

    def layer_end(self, layer: int, stream=None) -> int:
        return _check(lib().emoe_loader_layer_end(self._h, int(layer), _stream(stream)), "emoe_loader_layer_end", True)

    def layer_ready(self, layer: int) -> bool:
        """True if every load enqueued for the layer so far has finished on the GPU (does not block)."""
        ready = ctypes.c_int32(0)
        _check(lib().emoe_loader_layer_ready(self._h, int(layer), ctypes.byref(ready)), "emoe_loader_layer_ready", True)
        return bool(ready.value)

    def residents(self, layer: int):
        out = (ctypes.c_int32 * self._slots[layer])()
        _check(lib().emoe_loader_residents(self._h, int(layer), out), "emoe_loader_residents", True)
        return list(out)

    def synchronize(self) -> int:
        return _check(lib().emoe_loader_synchronize(self._h), "emoe_loader_synchronize", True)

    def close(self):
        if self._h:
            lib().emoe_loader_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class EmoeRequest(ctypes.Structure):
    _fields_ = [("input_tokens", ctypes.c_int32), ("g_remaining", ctypes.c_int32), ("g_initial", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("slo", ctypes.c_double), ("first_token_slo", ctypes.c_double),
                ("run_time", ctypes.c_double), ("delta_e", ctypes.c_double)]


def make_request(input_tokens, slo, first_token_slo, run_time=0.0, g_remaining=0, g_initial=0, delta_e=0.0) -> EmoeRequest:
    return EmoeRequest(int(input_tokens), int(g_remaining), int(g_initial), 0, float(slo), float(first_token_slo),
                       float(run_time), float(delta_e))


def _request_array(requests):
    requests = list(requests)
    return (EmoeRequest * max(len(requests), 1))(*requests), len(requests)


def emoe_expected_latency(running, i, c, new_request=None, check=True):
    arr, n = _request_array(running)
    out = ctypes.c_double(0.0)
    new = ctypes.byref(new_request) if new_request is not None else None
    rc = lib().emoe_expected_latency(n, arr, int(i), ctypes.c_double(c), new, ctypes.byref(out))
    _check(rc, "emoe_expected_latency", check)
    return out.value if rc == EMOE_OK else rc


def emoe_schedule(waiting, scheduled, t_max, c, check=True):
    """Indices of the admitted waiting requests, in admission order (or the status)."""
    w, nw = _request_array(waiting)
    s, ns = _request_array(scheduled)
    out = (ctypes.c_int32 * max(nw, 1))()
    n = ctypes.c_int32(0)
    rc = lib().emoe_schedule(nw, w, ns, s, ctypes.c_int64(int(t_max)), ctypes.c_double(c), out, ctypes.byref(n))
    _check(rc, "emoe_schedule", check)
    return list(out)[:n.value] if rc == EMOE_OK else rc


def emoe_generation_tick(request: EmoeRequest, completed: bool, reset_fraction: float = 0.05, check=True) -> int:
    rc = lib().emoe_generation_tick(ctypes.byref(request), 1 if completed else 0, ctypes.c_double(reset_fraction))
    return _check(rc, "emoe_generation_tick", check)
