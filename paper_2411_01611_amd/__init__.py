"""MI355X-native hot path of the skew-aware cached embedding-bag step (SCARS, arxiv 2411.01611).

`paper_2411_01611_amd.binding` is the ctypes binding over the C-ABI library built from `csrc/`;
`paper_2411_01611_amd.synth` draws seeded synthetic workloads and holds no method arithmetic.
"""
__all__ = ["binding", "synth"]
