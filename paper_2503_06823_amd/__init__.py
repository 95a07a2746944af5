"""Resident-expert MoE layer forward for AMD MI355X (gfx950): hand-written HIP kernels behind a
C ABI (include/emoe.h), plus this thin ctypes binding.  PyTorch is used by callers for device
memory and streams only."""
from .binding import (EMOE_ACT_RELU, EMOE_ACT_SWIGLU, EMOE_BF16, EMOE_ERR_DEVICE, EMOE_ERR_NULL, EMOE_ERR_RESIDENT,
                      EMOE_ERR_SHAPE, EMOE_ERR_UNSUPPORTED, EMOE_ERR_WORKSPACE, EMOE_F32, EMOE_OK, EXPORTS, LIB_PATH,
                      EmoeError, EmoeLayerDesc, emoe_combine, emoe_layer_forward, emoe_expert_ffn, emoe_expert_ffn_pass, emoe_expert_ffn_gather, emoe_expert_ffn_gather_pass, emoe_expert_ffn_gather_combine, emoe_load_experts, emoe_permute, emoe_permute_static,
                      emoe_measure_mfma_loop, emoe_measure_read_stream, emoe_measure_copy_stream, emoe_measure_scatter_combine,
                      emoe_route, emoe_route_observe, emoe_expected_latency, emoe_schedule, emoe_generation_tick, make_request,
                      EmoeRequest, emoe_prompt_action, Loader, EMOE_PROMPT_REUSE, EMOE_PROMPT_LOAD_ALL,
                      EMOE_PROMPT_PREDICT, emoe_expected_tokens, emoe_select_experts, emoe_plan_load,
                      emoe_workspace_bytes, lib, make_desc, make_event, status_string)
from .layer import DeviceInputs, LayerBuffers, layer_forward
