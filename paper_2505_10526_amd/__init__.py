"""MI355X (gfx950) implementation of the target-model verify step of
speculative decoding (Section 2.1 of the MASSV paper): verify_attention,
verify_layer, lm_head_logits and spec_accept as hand-written HIP kernels behind
a C ABI, with a ctypes binding in `binding`."""
