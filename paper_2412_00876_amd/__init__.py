"""MI355X-native sparsify-then-attend hot path of Dynamic-LLaVA (C-ABI library + ctypes binding)."""
from .binding import (BF16, F32, MODE_THRESHOLD, MODE_TOPK, PAGE_SIZE, DllavaError, KVCache,  # noqa: F401
                      dllava_decode_attn_append, dllava_decode_workspace, dllava_prefill_attn, dllava_score,
                      dllava_score_workspace, dllava_select_compact, dllava_select_compact_workspace,
                      dllava_version)
