"""The C-ABI library on a machine without a GPU: it loads, exports every symbol the header
declares, and rejects bad arguments on the host without enqueuing anything."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2503_06823_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built_library():
    if not os.path.exists(P.LIB_PATH):
        from paper_2503_06823_amd.build import build_library
        build_library(force=False)
    return P.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "emoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(emoe_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert sorted(P.EXPORTS) == names
    for n in names:
        assert getattr(P.lib(), n) is not None


def test_status_strings():
    seen = set()
    for code in range(0, -7, -1):
        s = P.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 7
    assert P.status_string(-99) == "unknown status"


def good(**kw):
    base = dict(T=64, d_model=128, d_ff=256, E=8, k=2, S=4, dtype="bf16", act="swiglu")
    base.update(kw)
    return P.make_desc(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=7), P.EMOE_ERR_UNSUPPORTED), (dict(act=5), P.EMOE_ERR_UNSUPPORTED),
    (dict(E=65, S=8), P.EMOE_ERR_UNSUPPORTED), (dict(d_model=100), P.EMOE_ERR_UNSUPPORTED),
    (dict(d_ff=12), P.EMOE_ERR_UNSUPPORTED), (dict(T=-1), P.EMOE_ERR_SHAPE), (dict(k=0), P.EMOE_ERR_SHAPE),
    (dict(k=5), P.EMOE_ERR_SHAPE), (dict(S=9), P.EMOE_ERR_SHAPE), (dict(d_model=0), P.EMOE_ERR_SHAPE),
    (dict(T=1 << 20, d_ff=1 << 14), P.EMOE_ERR_SHAPE),
])
def test_bad_descriptors_are_rejected_by_every_entry_point(kw, code):
    d = good(**kw)
    p = 4096  # a non-NULL address that must never be dereferenced
    assert P.emoe_workspace_bytes(d, check=False) == (code, code)
    assert P.emoe_route(d, p, p, None, p, p, p, stream=0, check=False) == code
    assert P.emoe_route_observe(d, p, p, None, p, p, p, p, stream=0, check=False) == code
    assert P.emoe_permute(d, p, p, p, p, p, p, p, p, p, 1 << 30, stream=0, check=False) == code
    assert P.emoe_expert_ffn(d, p, p, p, p, p, p, p, 1 << 30, stream=0, check=False) == code
    assert P.emoe_expert_ffn_gather(d, p, p, p, p, p, p, p, p, 1 << 30, stream=0, check=False) == code
    assert P.emoe_combine(d, p, p, p, p, stream=0, check=False) == code


def test_null_pointers_and_small_workspace():
    d = good()
    p = 4096
    pws, fws = P.emoe_workspace_bytes(d)
    assert pws > 0 and fws >= 64 * 2 * 256 * 2
    assert P.lib().emoe_workspace_bytes(None, None, None) == P.EMOE_ERR_NULL
    assert P.emoe_route(d, None, p, None, p, p, p, stream=0, check=False) == P.EMOE_ERR_NULL
    assert P.emoe_route(d, p, p, None, p, p, None, stream=0, check=False) == P.EMOE_ERR_NULL
    assert P.emoe_route_observe(d, p, p, None, p, p, p, None, stream=0, check=False) == P.EMOE_ERR_NULL
    assert P.emoe_permute(d, p, p, p, p, p, p, None, p, p, pws, stream=0, check=False) == P.EMOE_ERR_NULL
    assert P.emoe_permute(d, p, p, p, p, p, p, p, p, p, pws - 1, stream=0, check=False) == P.EMOE_ERR_WORKSPACE
    assert P.emoe_permute(d, p, p, p, p, p, p, p, p, None, pws, stream=0, check=False) == P.EMOE_ERR_WORKSPACE
    assert P.emoe_expert_ffn(d, p, p, p, None, p, p, p, fws, stream=0, check=False) == P.EMOE_ERR_NULL  # SwiGLU needs W3
    assert P.emoe_expert_ffn(good(act="relu"), p, p, p, p, p, p, p, fws, stream=0, check=False) == P.EMOE_ERR_UNSUPPORTED
    assert P.emoe_expert_ffn(d, p, p, p, p, p, p, p, fws - 1, stream=0, check=False) == P.EMOE_ERR_WORKSPACE
    assert P.emoe_expert_ffn_gather(d, p, None, p, p, p, p, p, p, fws, stream=0, check=False) == P.EMOE_ERR_NULL
    assert P.emoe_expert_ffn_gather(d, p, p, p, p, p, p, p, p, fws - 1, stream=0, check=False) == P.EMOE_ERR_WORKSPACE
    assert P.emoe_expert_ffn_gather_pass(d, 3, p, p, p, p, p, p, p, p, fws, stream=0, check=False) == P.EMOE_ERR_SHAPE
    assert P.emoe_combine(d, p, None, p, p, stream=0, check=False) == P.EMOE_ERR_NULL


def test_workspace_sizes_scale_with_the_layer():
    a = P.emoe_workspace_bytes(good(T=4096, d_model=4096, d_ff=14336))
    assert a[1] >= 4096 * 2 * 14336 * 2           # h: [A, f] bf16
    b = P.emoe_workspace_bytes(good(T=4096, d_model=4096, d_ff=14336, dtype="f32"))
    assert b[1] >= 4096 * 2 * 14336 * 4           # h in fp32
    assert all(v % 256 == 0 for v in a + b)


def test_ffn_workspace_holds_the_partial_sums_of_the_tile_paths():
    """The bf16 FFN takes one of three paths by the average rows per slot (A / S): up to 22 the
    streaming kernels (h only), up to 100 the 128-row tiles (h + 32 MiB of K pieces), above that
    the 256-row tiles (h + a 256-byte plan + 64 MiB); fp32 needs h only.  A layer whose weights are
    small is an exception to the last step."""
    def h_bytes(T, k, f, elem):
        return (T * k * f * elem + 255) // 256 * 256
    S, k, f = 4, 2, 256
    # a small layer takes the 128-row tiles again from 170 to 300 rows per slot
    for T, extra in ((44, 0), (45, 32 << 20), (200, 32 << 20), (201, 256 + (64 << 20)), (339, 256 + (64 << 20)),
                     (340, 32 << 20), (600, 32 << 20), (601, 256 + (64 << 20)), (4096, 256 + (64 << 20))):
        assert P.emoe_workspace_bytes(good(T=T, S=S, k=k, d_ff=f))[1] == h_bytes(T, k, f, 2) + extra, T
    assert P.emoe_workspace_bytes(good(T=4096, S=S, k=k, d_ff=f, dtype="f32"))[1] == h_bytes(4096, k, f, 4)


def load_args(d, eos_host):
    E = d.E
    w = [np.zeros(8, dtype=np.uint16) for _ in range(E)]
    return dict(host_w1=w, host_w3=w, host_w2=w, w1_slots=4096, w3_slots=4096, w2_slots=4096, slot_of_expert=4096,
                expert_of_slot=4096, expert_of_slot_host=eos_host, side_stream=0)


@pytest.mark.parametrize("experts,slots", [
    ([8], [0]),            # expert id out of range
    ([-2], [0]),           # below "empty"
    ([1], [4]),            # slot id out of range
    ([1, 2], [0, 0]),      # slot named twice
    ([1, 1], [0, 1]),      # expert named twice
    ([-1, -1, -1], [0, 1, 2]),  # would leave 1 resident expert, fewer than k = 2
])
def test_load_experts_rejects_bad_lists_and_leaves_the_mirror_alone(experts, slots):
    d = good()
    eos = np.array([0, 3, 5, 6], dtype=np.int32)
    before = eos.copy()
    rc = P.emoe_load_experts(d, experts, slots, **load_args(d, eos), check=False)
    assert rc == P.EMOE_ERR_RESIDENT
    assert np.array_equal(eos, before)


def test_load_experts_rejects_missing_host_weights_and_bad_mirror():
    d = good()
    eos = np.array([0, 3, 5, 6], dtype=np.int32)
    args = load_args(d, eos)
    args["host_w2"] = [None] * d.E
    assert P.emoe_load_experts(d, [1], [0], **args, check=False) == P.EMOE_ERR_NULL
    bad = np.array([0, 0, 5, 6], dtype=np.int32)          # mirror holds expert 0 twice
    assert P.emoe_load_experts(d, [1], [3], **load_args(d, bad), check=False) == P.EMOE_ERR_RESIDENT
    assert P.emoe_load_experts(d, [1] * 5, [0] * 5, **load_args(d, eos), check=False) == P.EMOE_ERR_SHAPE
