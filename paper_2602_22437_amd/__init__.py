"""MI355X-native RaggedShard / DBuffer hot path: thin ctypes binding over libraggedshard.so.

All arithmetic runs in the HIP library; this package only marshals arguments.  Importing
`paper_2602_22437_amd.binding` fails loudly when the library has not been built
(`python -m paper_2602_22437_amd.build` or `__graft_entry__.build()`).
"""
__all__ = ["binding", "build"]
