"""MI355X-native search path of sparsity-aware IVF-PQ (JUNO, arxiv 2312.01712).

`binding` holds the thin ctypes front end of the C-ABI library built from
`csrc/`; `workloads` holds the seeded synthetic inputs and the offline trainer.
"""
