"""LoMA attention hot path for MI355X (gfx950): hand-written HIP kernels behind a C ABI.

`paper_2401_09486_amd.loma` is the thin binding over the shared library (`loma_mask_attn_fwd`, `loma_mask_attn_bwd`,
`loma_compress_step`, `loma_decode_attn` and its layered, grouped-query, rotary and no-workspace forms,
`loma_prefill_attn`, the position-id helpers);
`paper_2401_09486_amd.workloads` draws the seeded synthetic inputs.
"""
__all__ = ["loma", "workloads"]
