"""MI355X-native NVFP4 hot path: quantizer, block-scaled FP4 GEMM, KV cache (HIP, gfx950)."""
from .binding import (LORA_RANK, KV_MAX_CHUNKS, ACT_GELU_TANH, ACT_NONE, OP_GEMM, OP_GEMM_ACT_QUANT, OP_GEMM_ACT_QUANT_GEMM, OP_GEMM_LORA, OP_LORA_DOWN, OP_KV_DEQUANT, OP_KV_QUANT, OP_KV_QUANT_4OVER6, OP_KV_QUANT_K, OP_KV_DEQUANT_GATHER, OP_QUANTIZE, OP_QUANTIZE_2D, OP_QUANTIZE_A2A, OP_QUANTIZE_RHT, OP_QUANTIZE_4OVER6, OUT_BF16,
                      OUT_F32, NVFP4Error, NVFP4Tensor, bf16_from_bits, bits_from_bf16, lib,
                      nvfp4_gemm, nvfp4_gemm_act_quant, nvfp4_gemm_lora, nvfp4_gemm_plan, nvfp4_lora_down, nvfp4_kv_dequant, nvfp4_kv_quant, nvfp4_kv_quant_4over6, nvfp4_kv_quant_noalloc, NOALLOC_MAX_ELEMENTS, nvfp4_kv_quant_k, nvfp4_kv_dequant_gather,
                      nvfp4_quantize, nvfp4_quantize_2d, nvfp4_quantize_for_all_to_all, nvfp4_quantize_rht, nvfp4_quantize_4over6, nvfp4_set_timing, nvfp4_set_timing_ops, nvfp4_timing_read, nvfp4_timing_read_all, nvfp4_workspace_bytes,
                      OP_PROBE, OP_GEMM_SCALE_OUT, nvfp4_gemm_scale_out, nvfp4_probe, nvfp4_set_sync_spin_limit, PROBE_READ, PROBE_WRITE, PROBE_COPY, PROBE_MFMA, PROBE_MFMA_FLOPS_PER_ITER)
