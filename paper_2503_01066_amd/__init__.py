"""MI355X-native hot path of activation-reuse training (capture/pack + backward from saved
activations).  The arithmetic lives in libalch.so (HIP, gfx950); this package only marshals
arguments (binding) and moves records between host and device (offload).  See include/alch.h for
the contract of every entry point."""
from .binding import (AlchError, lib, library_path, Batch, DpoItems, make_shape, alch_capture_pack, alch_capture_pack_static, alch_capture_gather, alch_layer_backward,
                      alch_layer_backward_lora, alch_stack_backward, alch_stack_backward_lora, alch_stack_backward_dpo, alch_layer_forward,
                      alch_gemm, alch_attention_forward, alch_trace_enable, alch_trace_collect,
                      layer_backward_workspace_bytes, stack_backward_workspace_bytes, PROJECTIONS, RECORD_KEYS,
                      WEIGHT_KEYS, STATUS)
from .offload import RecordStore
