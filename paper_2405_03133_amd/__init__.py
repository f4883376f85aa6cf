"""MI355X-native Lory causal-segment expert-merging MoE FFN layer.

The compute lives in the HIP library under csrc/ behind the C ABI declared in
include/lory.h; `binding` marshals torch device pointers into it.
"""
