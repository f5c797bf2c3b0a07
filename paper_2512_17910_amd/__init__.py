"""MI355X-native masked multi-adapter aLoRA QKV projection + paged K/V write.

`paper_2512_17910_amd.binding` is the thin Python layer over the C-ABI library built from
`csrc/`; `paper_2512_17910_amd.workloads` draws seeded synthetic inputs.  Nothing is imported
eagerly so that the input generators can be used without the HIP library.
"""
__all__ = ["binding", "workloads"]
