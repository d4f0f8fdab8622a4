"""MI355X linear attention (kernel a + b*x): thin Python binding over libla.so.

Every step of the computation runs in the HIP library; this package only
marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import (EXPORTS, LA_BF16, LA_F32, LA_MAX_TRACE, LaError, la_backward,
                      la_debug_override, la_forward_static, LA_STATIC_SCRATCH_BYTES,
                      la_decode_state_bytes, la_decode_step, la_decode_prefill, la_backward_ab, la_forward_qknorm, la_backward_qknorm,
                      la_forward_qknorm_save, la_backward_qknorm_saved,
                      la_backward_saved, la_backward_traced, la_forward, la_forward_save,
                      la_forward_traced, la_saved_state_bytes, la_status_string, la_trace,
                      la_version, la_workspace_bytes, library_path, load_library)

from .autograd import LinearAttentionFunction, linear_attention

__all__ = ["LinearAttentionFunction", "linear_attention", "LA_F32", "LA_BF16", "LA_MAX_TRACE", "EXPORTS", "LaError", "la_forward", "la_backward",
           "la_forward_traced", "la_backward_traced", "la_forward_save", "la_backward_saved",
           "la_saved_state_bytes", "la_trace", "la_debug_override", "la_decode_state_bytes", "la_decode_step", "la_decode_prefill", "la_backward_ab", "la_forward_qknorm", "la_backward_qknorm", "la_forward_qknorm_save", "la_backward_qknorm_saved", "la_forward_static", "LA_STATIC_SCRATCH_BYTES", "la_workspace_bytes",
           "la_status_string", "la_version", "library_path", "load_library"]
