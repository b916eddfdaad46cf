"""MI355X-native erasure-code hot path of GhostServe's shadow checkpointing.

`paper_2605_00831_amd.binding` wraps the C-ABI HIP library (include/ghostserve_ec.h);
`paper_2605_00831_amd.inputs` holds the seeded synthetic workloads.  The library
is loaded on first use of the binding and its absence is a hard error.
"""
