"""MI355X-native LazyAR beam decode for multi-level semantic-ID generation.

`paper_2602_22732_amd.binding` loads the HIP library (C ABI in include/gr4ad.h);
`paper_2602_22732_amd.synth` draws the seeded synthetic workloads.  Nothing is
imported eagerly, so the workload generator can be used without a built library.
"""
__all__ = ["binding", "synth"]
