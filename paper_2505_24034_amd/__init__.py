"""MI355X-native AIPO hot path (token log-probs + off-policy loss, fwd/bwd).

The compute lives in csrc/ (HIP for gfx950) behind the C ABI declared in
include/llamarl.h; `binding` marshals torch device pointers into it.
"""
