"""MI355X-native verify+draft attention and lossless acceptance (FlexDraft hot path).

`paper_2605_20022_amd.flexdraft` is the thin ctypes binding over the C-ABI library
built from `csrc/`; `paper_2605_20022_amd.workloads` draws seeded synthetic inputs.
"""
