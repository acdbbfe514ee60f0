"""MI355X-native hot path of spatial-temporal prefill/decode sharing (arXiv 2504.19516).

`paper_2504_19516_amd.synth`  seeded synthetic inputs (no method arithmetic)
`paper_2504_19516_amd.sts`    ctypes binding of the C-ABI library `libsts.so` (loaded on first use)
"""
__all__ = ["synth", "sts"]
