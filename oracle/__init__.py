"""CPU oracle for the FlexDraft verify+draft hot path.

TEST INFRASTRUCTURE ONLY.  This package is the slow, definition-level fp64
statement of what the HIP library must compute.  It may be imported by
`tests/`, by `__graft_entry__.smoke()` and by the `cpu_baseline` leg of
`bench.py`; nothing in `paper_2605_20022_amd/` imports it, and it imports
nothing from there.  It shares no code, tables or helpers with the HIP path.
"""
