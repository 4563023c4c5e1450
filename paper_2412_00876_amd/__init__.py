"""MI355X-native sparsify-then-attend hot path of Dynamic-LLaVA (C-ABI library + ctypes binding).

The binding (and with it the shared library) is loaded on first use of any of its names, so that the build
module can be imported before the library exists.  There is no fallback: without the built library the first
use raises ImportError.
"""
_BINDING_NAMES = ("BF16", "F32", "MODE_THRESHOLD", "MODE_THRESHOLD_KEEP_LAST", "MODE_TOPK", "PAGE_SIZE", "DllavaError", "KVCache", "EXPORTS",
                  "dllava_decode_attn_append", "dllava_decode_workspace", "dllava_prefill_attn", "dllava_score",
                  "dllava_score_workspace", "dllava_qkv_project", "dllava_decode_step", "dllava_decode_step_workspace",
                  "dllava_decode_commit", "dllava_predict", "dllava_predict_workspace", "Predictor", "dllava_linear", "dllava_layer_norm",
                  "dllava_span_attn", "dllava_masked_attn", "dllava_masked_attn_workspace", "dllava_compact", "dllava_rms_norm", "dllava_linear_few", "dllava_linear_few_workspace", "dllava_rope", "dllava_qkv_few", "dllava_gated_few", "dllava_decode_proj_workspace",
                  "dllava_select_compact", "dllava_select_compact_workspace", "dllava_version", "lib",
                  "dllava_set_launch_override", "dllava_decode_attn_append_static", "LAUNCH_DECODE_WAVES", "LAUNCH_DECODE_SPLITS", "LAUNCH_PREFILL_WAVES", "LAUNCH_SCORE_TILE", "LAUNCH_QKV_TILE", "LAUNCH_PREFILL_BLOCKS",
                  "LAUNCH_SELECT_LAUNCHES")


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_BINDING_NAMES))
