"""AGoQ quantization hot path for AMD MI355X: thin Python binding over libagoq.so.

The functions below marshal torch device tensors into the C ABI declared in
include/agoq.h (same names without the prefix).  Every step of the method runs in the
HIP kernels of that library; there is no fallback: without the built library, or
without a GPU, the calls raise.
"""
from .binding import (AgoqError, ActSlot, LayerSlots, MAX_LAYER_SLOTS, act_dequant, act_dequant_layer, act_quant_layer, layer_slots, act_dequant_rmsnorm, act_dequant_silu_mul, act_quant, codes_bytes, dbca_bits,
                      dbca_stored_microbatches, fp4_act_dequant, fp4_act_quant, fp8_grad_dequant,
                      fp8_grad_accumulate, fp8_grad_quant, fp8_grad_reduce_requant, grad_accumulate, grad_dequant, grad_quant,
                      grad_reduce_requant, rmsnorm_fwd_quant, silu_mul_fwd_quant,
                      layer_bitmap, layer_stored_bytes, library_path, load_library,
                      num_groups, strerror, version)

__all__ = [
    "AgoqError", "ActSlot", "LayerSlots", "MAX_LAYER_SLOTS", "act_quant", "act_dequant", "act_quant_layer", "act_dequant_layer", "layer_slots", "grad_quant", "grad_reduce_requant",
    "grad_accumulate", "grad_dequant", "fp4_act_quant", "fp4_act_dequant", "fp8_grad_quant",
    "fp8_grad_dequant", "fp8_grad_reduce_requant", "fp8_grad_accumulate", "act_dequant_rmsnorm", "act_dequant_silu_mul", "rmsnorm_fwd_quant", "silu_mul_fwd_quant",
    "codes_bytes", "num_groups", "dbca_bits", "dbca_stored_microbatches", "layer_bitmap",
    "layer_stored_bytes", "strerror", "version", "load_library", "library_path",
]
