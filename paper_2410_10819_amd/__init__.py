"""MI355X-native DuoAttention hot path: split KV cache + prefill/decode attention kernels.

The compute lives in csrc/ (HIP for gfx950) behind the C-ABI declared in
include/duoattn.h; `binding` marshals arguments to it and `synth` makes inputs.
"""
