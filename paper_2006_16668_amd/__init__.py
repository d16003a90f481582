"""MI355X-native forward pass of GShard's top-2 Mixture-of-Experts layer.

``binding`` holds thin ctypes wrappers around the C ABI declared in
``include/moe_gfx950.h``; every step of the layer runs in the HIP kernels of
``libmoe_gfx950.so`` (built by ``python -m paper_2006_16668_amd.build``).
There is no CPU fallback: a missing library raises on first use.
"""
from .binding import (EncoderDims, moe_add_layer_norm, moe_attention_workspace_bytes,
                      moe_dense_ffn, moe_encoder_pair_forward, moe_encoder_workspace_bytes,
                      moe_encoder_pair_forward_train, moe_encoder_pair_backward,
                      moe_encoder_train_workspace_bytes, moe_encoder_backward_workspace_bytes,
                      moe_self_attention, moe_backward, moe_backward_events, moe_backward_workspace_bytes,
                      moe_forward_train, MoEError, MoEShape, library_path, load_library, moe_combine, moe_dispatch,
                      moe_expert_ffn, moe_expert_ffn_workspace_bytes, moe_forward_packs_rows, moe_forward, moe_forward_events, moe_forward_fuses_dispatch,
                      moe_gate, moe_gate_pack, moe_gate_pack_bytes, moe_gate_prepacked, moe_forward_prepacked, moe_gate_noalloc, moe_gate_noalloc_max_bytes, moe_gate_workspace_bytes,
                      moe_prepare, moe_status_string, moe_train_workspace_bytes, moe_workspace_bytes)

__all__ = ["EncoderDims", "moe_add_layer_norm", "moe_attention_workspace_bytes", "moe_dense_ffn",
           "moe_encoder_pair_forward", "moe_encoder_workspace_bytes", "moe_self_attention",
           "moe_encoder_pair_forward_train", "moe_encoder_pair_backward",
           "moe_encoder_train_workspace_bytes", "moe_encoder_backward_workspace_bytes",
           "moe_backward", "moe_backward_events", "moe_backward_workspace_bytes",
           "moe_forward_train", "MoEError", "MoEShape", "library_path", "load_library", "moe_combine", "moe_dispatch",
           "moe_expert_ffn", "moe_expert_ffn_workspace_bytes", "moe_forward_packs_rows", "moe_forward", "moe_forward_events", "moe_forward_fuses_dispatch",
           "moe_gate", "moe_gate_pack", "moe_gate_pack_bytes", "moe_gate_prepacked", "moe_forward_prepacked", "moe_gate_noalloc", "moe_gate_noalloc_max_bytes", "moe_gate_workspace_bytes",
           "moe_prepare", "moe_status_string", "moe_train_workspace_bytes", "moe_workspace_bytes"]
