"""MI355X-native filtered int8 top-K retrieval (Bloom index + int8 scoring + top-K).

`paper_2511_14881_amd.binding` is the Python face of the C-ABI library built from
`csrc/`; `paper_2511_14881_amd.synth` draws seeded synthetic workloads.  Importing
the package loads nothing native: the library is opened on first use and raises
if it has not been built.
"""
__all__ = ["binding", "synth"]
