"""MI355X-native speculative decoding with a dynamic draft tree (the decode path of HASS / EAGLE-2).

The product is libspec.so (hand-written gfx950 kernels behind a C ABI, see include/spec.h); this
package is the thin ctypes binding over it.  Importing the binding without a built library raises.
"""
from .binding import (Engine, SpecError, Tree, lib, spec_accept, spec_committed, spec_create, spec_destroy, spec_draft_tree,
                      spec_get_features, spec_get_kv, spec_hca_attention, spec_topk_loss, spec_topk_loss_scratch_bytes, spec_get_logits, spec_get_profile, spec_k_accept_qratio, spec_k_attention, spec_k_gemm, spec_k_gemm_swiglu, spec_k_sample_children,
                      spec_k_topk_logprob, spec_k_topk_logprob_static, spec_last_error, spec_pack_gate_up, spec_pack_weight, spec_packed_bytes, spec_prefill, spec_set_graphs, spec_set_profile, spec_verify,
                      spec_workspace_bytes, pack_weights, upload_weights)

__all__ = [n for n in dir() if not n.startswith("_")]
