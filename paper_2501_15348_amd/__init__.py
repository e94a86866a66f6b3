"""MI355X-native hot path of incremental dynamic-GNN training (ReInc, arXiv 2501.15348).

`paper_2501_15348_amd.synth`  seeded synthetic inputs (numpy only)
`paper_2501_15348_amd.reinc`  thin ctypes binding over the C-ABI library `libreinc_hip.so`
"""
__all__ = ["synth", "reinc"]
