"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same seeded
inputs.  Index work must be bit-exact, gate weights within 1e-5, outputs within relative L2 1e-2
(bf16 storage, fp32 accumulation) or 1e-5 (fp32)."""
import numpy as np
import pytest
import torch

import emoe_inputs as gen
import oracle
import paper_2503_06823_amd as P
from gpu_util import (DeviceLayer, check_ffn_rows, check_outputs, check_routing_and_permutation, desc_of,
                      stratified_rows, to_dev)

pytestmark = pytest.mark.gpu


def cfg(name, **kw):
    base = dict(name=name, index=40, T=64, d_model=128, d_ff=256, E=8, k=2, R=4, dtype="bf16", act="swiglu")
    base.update(kw)
    return gen.LayerConfig(**base)


# Oracle-sized cases.  Each spans several tiles of the kernel it exercises and has a ragged tail.
SMALL_CASES = [
    gen.C1,                                                                       # fp32 path, as specified
    cfg("f32_ragged", dtype="f32", T=150, d_model=72, d_ff=136, E=8, k=2, R=5, S=7, index=41),
    cfg("f32_relu_top1", dtype="f32", act="relu", T=97, d_model=64, d_ff=200, E=16, k=1, R=6, zipf_s=1.1, index=42),
    # tiles of 128 token rows (22 S < A <= 100 S): slots of less than one tile and (the skewed ones) of
    # several, N tails, K tail (d=328, f=456 not % 64), empty slots, top-6
    cfg("mid_swiglu_ragged", T=190, d_model=328, d_ff=456, E=8, k=2, R=4, index=43),
    cfg("mid_swiglu_aligned", T=240, d_model=512, d_ff=768, E=8, k=2, R=3, S=5, index=44),
    cfg("mid_relu_skewed", act="relu", T=1500, d_model=256, d_ff=520, E=64, k=1, R=16, zipf_s=1.1, index=45),
    cfg("mid_long_k_ktail", T=280, d_model=1032, d_ff=1160, E=8, k=2, R=4, S=6, index=58),
    cfg("mid_topk6", T=380, d_model=256, d_ff=384, E=64, k=6, R=24, zipf_s=1.2, resident="popular", index=46),
    # enough output tiles that the first product takes tiles of 256 weight rows (all other small cases take 128)
    cfg("mid_relu_wide_ff", act="relu", T=1500, d_model=72, d_ff=2560, E=64, k=1, R=16, zipf_s=1.1, index=66),
    cfg("mid_swiglu_wide_ff", T=800, d_model=72, d_ff=1408, E=16, k=2, R=16, index=67),
    cfg("mid_few_rows_per_slot", T=100, d_model=192, d_ff=264, E=8, k=2, R=5, index=60),
    # 29-48 rows per slot and more tiles than CUs: token tiles of 64 rows (K tail, N tail, slots of 0 to 3 tiles)
    cfg("mid_64_row_tiles_swiglu", T=320, d_model=72, d_ff=1792, E=16, k=2, R=16, index=72),
    cfg("mid_64_row_tiles_relu", act="relu", T=640, d_model=136, d_ff=3336, E=64, k=1, R=16, zipf_s=1.1, index=73),
    # a long K and fewer 128 x 128 tiles than CUs: the persistent launch cuts the tiles along K and a second kernel
    # adds the pieces (first product: K = 4104 with a K tail; second product: K = 4160)
    cfg("mid_cut_first_product", T=100, d_model=4104, d_ff=264, E=8, k=2, R=3, index=68),
    cfg("mid_cut_second_product", act="relu", T=240, d_model=200, d_ff=4160, E=8, k=1, R=4, index=69),
    # the same with at most 48 rows per slot: 64-row token tiles in the persistent launch (plain and ReLU products)
    cfg("mid_64_row_cut_second_product", T=80, d_model=200, d_ff=4160, E=8, k=2, R=4, index=74),
    cfg("mid_64_row_cut_first_product_relu", act="relu", T=160, d_model=4104, d_ff=264, E=8, k=1, R=4, index=75),
    # a long K and about as many tiles as CUs, or more: the persistent launch takes whole tiles, one or two each
    cfg("mid_persistent_whole_tiles", T=300, d_model=4096, d_ff=1152, E=8, k=2, R=8, index=70),
    cfg("mid_persistent_two_rounds", act="relu", T=1600, d_model=4096, d_ff=2048, E=64, k=1, R=16, zipf_s=1.1, index=71),
    # tiles of 256 token rows (A > 100 S): several M tiles + tail, N tails, K tail
    cfg("tiled_swiglu_ragged", T=1700, d_model=328, d_ff=456, E=8, k=2, R=4, index=61),
    cfg("tiled_swiglu_aligned", T=1024, d_model=512, d_ff=768, E=8, k=2, R=3, S=5, index=62),
    cfg("tiled_relu_skewed", act="relu", T=6400, d_model=256, d_ff=520, E=64, k=1, R=16, zipf_s=1.1, index=63),
    # few output tiles and a long K: leftover tiles are split along K into pieces (with a K tail in both passes)
    cfg("tiled_splitk_ktail", T=800, d_model=1032, d_ff=1160, E=8, k=2, R=4, index=64),
    cfg("tiled_topk6", T=1600, d_model=256, d_ff=384, E=64, k=6, R=24, zipf_s=1.2, resident="popular", index=65),
    # streaming path (A <= 22 S): few rows per slot, slots with 0 rows, a slot with > 64 rows
    cfg("stream_decode", T=64, d_model=512, d_ff=1088, E=8, k=2, R=6, index=47),
    cfg("stream_ktail", T=20, d_model=200, d_ff=328, E=8, k=2, R=5, S=8, index=48),
    cfg("stream_relu_hot_slot", act="relu", T=88, d_model=256, d_ff=384, E=4, k=1, R=2, S=4, zipf_s=3.0, index=49),
    cfg("stream_two_token_blocks", T=80, d_model=128, d_ff=192, E=4, k=1, R=2, S=4, index=57),
    cfg("stream_k_equals_R", T=9, d_model=128, d_ff=192, E=6, k=3, R=3, index=50),
    # few tokens, few experts, long rows: the bf16 route that puts one workgroup on each token (d_model with a K tail)
    cfg("decode_long_rows", T=40, d_model=2056, d_ff=192, E=12, k=2, R=7, S=9, index=59),
    # many experts per token: top-8 of 12 resident (streaming and tiles), top-16 with every slot taken
    cfg("top8_of_12", T=40, d_model=128, d_ff=192, E=16, k=8, R=12, index=83),
    cfg("top8_of_12_tiles", T=300, d_model=200, d_ff=264, E=16, k=8, R=12, S=14, index=84),
    cfg("top16_all_slots", act="relu", T=150, d_model=128, d_ff=136, E=32, k=16, R=16, zipf_s=1.1, index=85),
    # more than 65 536 assignments: the permutation's three-launch path (scan as a launch of its own)
    cfg("permute_many_chunks", T=35000, d_model=64, d_ff=72, E=16, k=2, R=5, zipf_s=1.1, index=86),
    # expert counts that fill no group of 8, 16 or 32 gate rows
    cfg("experts_5", T=130, d_model=136, d_ff=200, E=5, k=2, R=3, S=4, index=87),
    cfg("experts_24", act="relu", T=260, d_model=200, d_ff=264, E=24, k=3, R=11, S=20, zipf_s=1.1, index=88),
    cfg("experts_48_decode", T=48, d_model=2056, d_ff=136, E=48, k=4, R=30, S=40, index=89),
    cfg("single_token", T=1, d_model=128, d_ff=256, E=8, k=2, R=4, index=51),
    cfg("single_expert_dense", T=300, d_model=128, d_ff=256, E=1, k=1, R=1, index=52),
]


@pytest.mark.parametrize("c", SMALL_CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("shuffle", [False, True], ids=["slots_in_order", "slots_shuffled"])
def test_layer_matches_oracle(gpu_device, c, shuffle):
    if shuffle and c.slots == 1:
        pytest.skip("one slot cannot be shuffled")
    inp = gen.make_layer_inputs(c, shuffle_slots=shuffle)
    ref = oracle.layer_forward(inp)
    dl = DeviceLayer(inp)
    dl.forward()
    torch.cuda.synchronize()
    check_routing_and_permutation(dl, ref)
    check_outputs(dl, ref)
    # the intermediate h as well, element by element (all rows of a small case)
    A = c.T * c.k
    if A > 0:
        rows = np.arange(A) if A <= 4096 else stratified_rows(ref.permutation.slot_offsets, c.seed)
        check_ffn_rows(dl, ref.permutation, rows)
    dl.check_gather_path_is_identical()


def test_each_call_alone_on_oracle_inputs(gpu_device):
    """Each entry point fed with the oracle's results for the steps before it."""
    c = cfg("per_call", T=300, d_model=256, d_ff=384, E=8, k=2, R=4, index=53)
    inp = gen.make_layer_inputs(c, shuffle_slots=True)
    ref = oracle.layer_forward(inp)
    dl = DeviceLayer(inp)
    b, d = dl.buf, dl.desc
    pm = ref.permutation
    # permute from the oracle's routing
    te = torch.from_numpy(ref.topk_expert).cuda()
    P.emoe_permute(d, dl.x, te, dl.slot_of_expert, b.slot_counts, b.slot_offsets, b.perm, b.inv_perm, b.x_perm,
                   b.permute_ws, b.permute_ws.numel())
    torch.cuda.synchronize()
    assert np.array_equal(b.perm.cpu().numpy(), pm.perm) and np.array_equal(b.inv_perm.cpu().numpy(), pm.inv_perm)
    # FFN from the oracle's x_perm / offsets
    xp = to_dev(oracle.gather_rows(inp.x, pm.perm, c.k, c.dtype), c.dtype)
    off = torch.from_numpy(pm.slot_offsets).cuda()
    P.emoe_expert_ffn(d, xp, off, dl.w1, dl.w3, dl.w2, b.y_perm, b.ffn_ws, b.ffn_ws.numel())
    # combine from the oracle's weights and inverse permutation
    tw = torch.from_numpy(ref.topk_weight.astype(np.float32)).cuda()
    ip = torch.from_numpy(pm.inv_perm).cuda()
    P.emoe_combine(d, b.y_perm, ip, tw, b.out)
    torch.cuda.synchronize()
    check_outputs(dl, ref)


def test_zero_tokens_is_a_noop(gpu_device):
    c = cfg("empty", T=0, index=54)
    d = desc_of(c)
    buf = P.LayerBuffers.allocate(d)
    buf.slot_counts.fill_(7)
    buf.slot_offsets.fill_(7)
    dummy = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    soe = torch.zeros(c.E, dtype=torch.int32, device="cuda")
    assert P.emoe_route(d, dummy, dummy, None, soe, buf.topk_expert, buf.topk_weight) == P.EMOE_OK
    assert P.emoe_permute(d, dummy, buf.topk_expert, soe, buf.slot_counts, buf.slot_offsets, buf.perm, buf.inv_perm,
                          buf.x_perm, buf.permute_ws, buf.permute_ws.numel()) == P.EMOE_OK
    assert P.emoe_expert_ffn(d, buf.x_perm, buf.slot_offsets, dummy, dummy, dummy, buf.y_perm, buf.ffn_ws,
                             buf.ffn_ws.numel()) == P.EMOE_OK
    assert P.emoe_combine(d, buf.y_perm, buf.inv_perm, buf.topk_weight, buf.out) == P.EMOE_OK
    assert P.emoe_expert_ffn_gather_combine(d, dummy, buf.perm, buf.inv_perm, buf.slot_offsets, dummy, dummy, dummy,
                                            buf.topk_weight, buf.y_perm, buf.out, buf.ffn_ws, buf.ffn_ws.numel()) == P.EMOE_OK
    torch.cuda.synchronize()
    assert not buf.slot_counts.cpu().numpy().any() and not buf.slot_offsets.cpu().numpy().any()
    buf.slot_counts.fill_(7)
    buf.slot_offsets.fill_(7)
    assert P.emoe_permute_static(d, dummy, buf.topk_expert, soe, buf.slot_counts, buf.slot_offsets, buf.perm, buf.inv_perm,
                                 buf.x_perm) == P.EMOE_OK
    torch.cuda.synchronize()
    assert not buf.slot_counts.cpu().numpy().any() and not buf.slot_offsets.cpu().numpy().any()


def test_results_are_reproducible_run_to_run(gpu_device):
    c = cfg("determinism", T=700, d_model=256, d_ff=384, E=16, k=2, R=6, zipf_s=1.1, index=55)
    dl = DeviceLayer(gen.make_layer_inputs(c))
    snaps = []
    for _ in range(5):
        dl.forward()
        torch.cuda.synchronize()
        b = dl.buf
        snaps.append([t.clone() for t in (b.topk_expert, b.topk_weight, b.perm, b.inv_perm, b.slot_offsets, b.y_perm,
                                          b.out)])
    for s in snaps[1:]:
        for t0, t1 in zip(snaps[0], s):
            assert torch.equal(t0, t1)


def test_all_experts_resident_equals_the_ordinary_layer(gpu_device):
    """First prompt of a session: every expert is on the GPU (Section 3.3)."""
    c = cfg("all_resident", T=200, d_model=128, d_ff=256, E=8, k=2, R=8, index=56)
    inp = gen.make_layer_inputs(c)
    ref = oracle.layer_forward(inp)
    assert np.array_equal(ref.topk_expert, oracle.route_unrestricted(ref.logits, c.k))
    dl = DeviceLayer(inp)
    dl.forward()
    torch.cuda.synchronize()
    check_routing_and_permutation(dl, ref)
    check_outputs(dl, ref)


def _random_cases(n, seed):
    """Seeded random small layers over every path: dtype, activation, extents with and without tails,
    few to many rows per slot, more slots than residents."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        dtype = "f32" if i % 6 == 5 else "bf16"
        act = "relu" if rng.random() < 0.3 else "swiglu"
        E = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
        R = int(rng.integers(1, E + 1))
        k = int(rng.integers(1, min(R, 6) + 1))
        S = int(rng.integers(R, E + 1))
        rows = int(rng.choice([3, 12, 30, 45, 70, 95, 110, 200, 420]))      # per slot, on average
        T = max(1, min(2500, rows * S // k))
        d_model = int(rng.choice([64, 72, 128, 200, 256, 328]))
        d_ff = int(rng.choice([64, 136, 192, 264, 520]))
        if dtype == "f32":
            T, d_model, d_ff = min(T, 300), min(d_model, 128), min(d_ff, 192)
        zipf = float(rng.choice([0.0, 0.0, 1.1]))
        cases.append(cfg(f"random{i}_{dtype}_{act}_T{T}_d{d_model}_f{d_ff}_E{E}_k{k}_R{R}_S{S}", dtype=dtype, act=act, T=T,
                         d_model=d_model, d_ff=d_ff, E=E, k=k, R=R, S=S, zipf_s=zipf, index=100 + i))
    return cases


@pytest.mark.parametrize("c", _random_cases(30, 20250306), ids=lambda c: c.name)
def test_random_small_layers(gpu_device, c):
    inp = gen.make_layer_inputs(c, shuffle_slots=c.index % 2 == 1 and c.slots > 1)
    ref = oracle.layer_forward(inp)
    dl = DeviceLayer(inp)
    dl.forward()
    torch.cuda.synchronize()
    check_routing_and_permutation(dl, ref)
    check_outputs(dl, ref)
    dl.check_gather_path_is_identical()


def _random_long_k_cases(n, seed):
    """Seeded random layers with one long and one short product (K >= 64 tiles of 64 in one of them)
    and 29-200 rows per slot: the persistent launch of the 128-row tiles, which cuts tiles along K
    when they are few, takes whole tiles otherwise, and the 256-row tiles' K pieces beyond that."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        act = "relu" if rng.random() < 0.3 else "swiglu"
        E = int(rng.choice([1, 2, 4, 8, 16]))
        R = int(rng.integers(1, E + 1))
        k = int(rng.integers(1, min(R, 4) + 1))
        S = int(rng.integers(R, E + 1))
        rows = int(rng.choice([29, 47, 64, 80, 100, 128, 200]))
        T = max(1, rows * S // k)
        big, small = int(rng.choice([4096, 4104, 4160, 6152])), int(rng.choice([64, 136, 264, 520]))
        d_model, d_ff = (big, small) if i % 2 == 0 else (small, big)
        cases.append(cfg(f"longk{i}_{act}_T{T}_d{d_model}_f{d_ff}_E{E}_k{k}_R{R}_S{S}", act=act, T=T, d_model=d_model,
                         d_ff=d_ff, E=E, k=k, R=R, S=S, index=200 + i))
    return cases


@pytest.mark.parametrize("c", _random_long_k_cases(12, 20250307), ids=lambda c: c.name)
def test_random_layers_with_a_long_k(gpu_device, c):
    inp = gen.make_layer_inputs(c, shuffle_slots=c.index % 2 == 1 and c.slots > 1)
    ref = oracle.layer_forward(inp)
    dl = DeviceLayer(inp)
    dl.forward()
    torch.cuda.synchronize()
    check_routing_and_permutation(dl, ref)
    check_outputs(dl, ref)
    dl.check_gather_path_is_identical()


# one expert per token on every FFN path: fp32, streaming, tiles of 64 / 128 / 256 token rows, whole and cut along K
TOP1_CASES = [c for c in SMALL_CASES if c.k == 1] + [
    cfg("tiled_top1_splitk", T=1600, d_model=1032, d_ff=1160, E=8, k=1, R=4, index=80),
    cfg("tiled_top1_swiglu_ragged", T=900, d_model=328, d_ff=456, E=8, k=1, R=3, S=4, index=81),
    cfg("mid_top1_swiglu", T=200, d_model=256, d_ff=384, E=8, k=1, R=4, index=82),
]


@pytest.mark.parametrize("c", TOP1_CASES, ids=lambda c: c.name)
def test_combine_folded_into_the_second_product(gpu_device, c):
    """k = 1: emoe_expert_ffn_gather_combine stores the second product's rows straight into `out`;
    bit for bit the result of emoe_expert_ffn_gather + emoe_combine, which the other tests compare
    with the oracle (and here once more)."""
    inp = gen.make_layer_inputs(c, shuffle_slots=c.slots > 1)
    ref = oracle.layer_forward(inp)
    dl = DeviceLayer(inp)
    dl.forward(gather_in_ffn=True)
    torch.cuda.synchronize()
    check_outputs(dl, ref)
    b, d = dl.buf, dl.desc
    separate = b.out.clone()
    b.out.fill_(float("nan"))
    y_before = b.y_perm.clone()
    P.emoe_expert_ffn_gather_combine(d, dl.x, b.perm, b.inv_perm, b.slot_offsets, dl.w1, dl.w3, dl.w2, b.topk_weight, None,
                                     b.out, b.ffn_ws, b.ffn_ws.numel())
    torch.cuda.synchronize()
    assert torch.equal(b.out.view(torch.int16) if b.out.dtype == torch.bfloat16 else b.out,
                       separate.view(torch.int16) if separate.dtype == torch.bfloat16 else separate)
    assert torch.equal(b.y_perm, y_before), "y_perm must stay untouched when the combine is folded in"


def test_folded_combine_with_several_experts_per_token_is_the_two_calls(gpu_device):
    c = [c for c in SMALL_CASES if c.name == "mid_swiglu_ragged"][0]
    dl = DeviceLayer(gen.make_layer_inputs(c))
    dl.forward(gather_in_ffn=True)
    torch.cuda.synchronize()
    b = dl.buf
    separate = b.out.clone()
    b.out.zero_(); b.y_perm.zero_()
    P.emoe_expert_ffn_gather_combine(dl.desc, dl.x, b.perm, b.inv_perm, b.slot_offsets, dl.w1, dl.w3, dl.w2, b.topk_weight,
                                     b.y_perm, b.out, b.ffn_ws, b.ffn_ws.numel())
    torch.cuda.synchronize()
    assert torch.equal(b.out, separate)
    rc = P.emoe_expert_ffn_gather_combine(dl.desc, dl.x, b.perm, b.inv_perm, b.slot_offsets, dl.w1, dl.w3, dl.w2,
                                          b.topk_weight, None, b.out, b.ffn_ws, b.ffn_ws.numel(), check=False)
    assert rc == P.EMOE_ERR_NULL        # with k > 1 y_perm is needed


@pytest.mark.parametrize("name", ["mid_swiglu_ragged", "mid_topk6", "tiled_swiglu_aligned"])
def test_combine_by_atomic_scatter_agrees_with_the_combine(gpu_device, name):
    """The measurement aid that does the combine the way a fold into the second product would (fp32
    atomics) computes the same output up to the rounding of a differently ordered fp32 sum."""
    c = [c for c in SMALL_CASES if c.name == name][0]
    dl = DeviceLayer(gen.make_layer_inputs(c))
    dl.forward(gather_in_ffn=True)
    b = dl.buf
    image = torch.empty((c.T, c.d_model), dtype=torch.float32, device="cuda")
    out2 = torch.full_like(b.out, float("nan"))
    P.emoe_measure_scatter_combine(dl.desc, b.y_perm, b.perm, b.topk_weight, image, out2)
    torch.cuda.synchronize()
    ref, got = b.out.double(), out2.double()
    assert torch.isfinite(got).all()
    # both round one fp32 sum of the same k products to bf16: at most one bf16 step apart
    assert ((got - ref).abs() <= 2.0 ** -7 * ref.abs() + 1e-5).all()


@pytest.mark.parametrize("name", ["mid_swiglu_ragged", "tiled_relu_skewed", "stream_decode", "C1_tiny_f32"])
def test_layer_forward_in_one_call_equals_the_four_calls(gpu_device, name):
    c = [c for c in SMALL_CASES if c.name == name][0]
    inp = gen.make_layer_inputs(c)
    a, b = DeviceLayer(inp), DeviceLayer(inp)
    P.layer_forward(a.buf, a.x, a.w_gate, a.gate_bias, a.slot_of_expert, a.w1, a.w3, a.w2, gather_in_ffn=True)
    P.layer_forward(b.buf, b.x, b.w_gate, b.gate_bias, b.slot_of_expert, b.w1, b.w3, b.w2, one_call=True)
    torch.cuda.synchronize()
    for f in ("topk_expert", "topk_weight", "slot_counts", "slot_offsets", "perm", "inv_perm", "y_perm", "out"):
        if f == "y_perm" and c.k == 1:
            continue        # one expert per token: the second product writes `out` directly, y_perm stays unwritten
        assert torch.equal(getattr(a.buf, f), getattr(b.buf, f)), f
    # an argument error is found before anything is enqueued: outputs stay as they are
    before = b.buf.out.clone()
    b.buf.out.zero_()
    rc = P.emoe_layer_forward(b.desc, b.x, b.w_gate, b.gate_bias, b.slot_of_expert, b.w1, b.w3, b.w2, b.buf.topk_expert,
                              b.buf.topk_weight, b.buf.slot_counts, b.buf.slot_offsets, b.buf.perm, b.buf.inv_perm,
                              b.buf.y_perm, b.buf.out, b.buf.permute_ws, b.buf.permute_ws.numel(), b.buf.ffn_ws,
                              b.buf.ffn_ws.numel() - 1, check=False)
    torch.cuda.synchronize()
    assert rc == P.EMOE_ERR_WORKSPACE
    assert not b.buf.out.any() and before.any()
