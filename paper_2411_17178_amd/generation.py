"""All KV-cache generation steps of one attention layer.

VAR generates scale by scale (paper Section 2): at step k the queries are the tokens of scale
k and the keys the tokens of scales 0..k, which the caller has appended to its K/V cache.  A
GenerationLayer holds one plan per step (query scales [k, k+1)) for a fixed cache layout
`[B, H, L, 64]` and enqueues the steps, one library call each, on the caller's stream.  With
`share_all` the unconditional half of the batch reuses the conditional half's attention
output in every head and at every scale (paper Section 3: the unconditional workgroups exit
at once, the conditional ones store both rows).

Argument marshalling only: the plans are built by litevar_mask_build and every step runs
litevar_windowed_attn_fwd (litevar_windowed_attn_qkv8_fwd for 8-bit caches).  The calls allocate nothing and never synchronise, so a caller may
capture them in a HIP graph (torch.cuda.graph) and replay a whole layer with one launch.
"""
import torch

from . import binding


class GenerationLayer:
    def __init__(self, scales, radius, radius_per_key_scale=None, n_sink_scales=0,
                 waves_per_group=0, device="cuda", batch_heads=0):
        self.scales = [int(s) for s in scales]
        self.offsets = binding.litevar_scale_offsets(self.scales)   # the library's scale table
        self.kv_len = self.offsets[-1]
        self.plans = [
            binding.litevar_mask_build(self.scales, radius, radius_per_key_scale, n_sink_scales,
                                       (k, k + 1), waves_per_group=waves_per_group, device=device,
                                       batch_heads=batch_heads)
            for k in range(len(self.scales))
        ]

    @property
    def n_steps(self):
        return len(self.plans)

    def rows(self, k):
        """Token range of scale k in the sequence (and in the caller's caches)."""
        return self.offsets[k], self.offsets[k + 1]

    def retained_pairs(self):
        return sum(int(p.retained_pairs) for p in self.plans)

    def step(self, k, q_k, k_cache, v_cache, sm_scale, out_k=None, share_all=False, stream=None):
        """Attention of scale k's queries `q_k` [B, H, s_k^2, 64] against the caches
        [B, H, L, 64]; only the rows of scales 0..k are read."""
        share = self._share_table(q_k) if share_all else None
        return binding.litevar_windowed_attn_fwd(self.plans[k], q_k, k_cache, v_cache, sm_scale,
                                                 out=out_k, cfg_share=share, stream=stream)

    def qkv8_workspace_bytes(self, B, H):
        """Bytes of the workspace that step_qkv8 needs at most (steps whose plan converts the
        8-bit operands in the attention kernel need none)."""
        return max(binding.litevar_windowed_attn_qkv8_workspace_bytes(p, B, H) for p in self.plans)

    def step_qkv8(self, k, q8_k, q_sz_k, k8_cache, k_sz_cache, v8_cache, v_sz_cache, sm_scale, out_k=None,
                  share_all=False, workspace=None, stream=None):
        """The same step on 8-bit operands (paper Section 4): codes int8 `[B, H, *, 64]` with one
        (scale, zero point) per token row, float32 `[B, H, *, 2]`, as litevar_qkv8_quantize
        returns them; the caches hold the rows of scales 0..k.  Packed tensors.  `workspace`:
        a uint8 CUDA tensor of qkv8_workspace_bytes() bytes (allocated per call when omitted)."""
        share = self._share_table(q8_k) if share_all else None
        return binding.litevar_windowed_attn_qkv8_fwd(self.plans[k], q8_k, q_sz_k, k8_cache, k_sz_cache,
                                                      v8_cache, v_sz_cache, sm_scale, out=out_k,
                                                      cfg_share=share, workspace=workspace, stream=stream)

    def prepare(self, q_steps, k_cache, v_cache, sm_scale, out_steps, share_all=False, stream=None):
        """Marshal all steps once; returns zero-argument callables, one per step, that
        enqueue the step (for launch-rate-sensitive loops and graph capture)."""
        share = self._share_table(q_steps[0]) if share_all else None
        return [binding.prepare_attn_call(self.plans[k], q_steps[k], k_cache, v_cache, sm_scale,
                                          out_steps[k], cfg_share=share, stream=stream)
                for k in range(self.n_steps)]

    def _share_table(self, q):
        H = q.shape[1]
        key = (H, q.device)
        if getattr(self, "_share_key", None) != key:
            self._share = torch.ones((H, len(self.scales)), dtype=torch.uint8, device=q.device)
            self._share_key = key
        return self._share
