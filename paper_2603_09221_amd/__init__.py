"""Batched finite-horizon LQR (Test-Time Control layer hot path) for AMD MI355X (gfx950).

`paper_2603_09221_amd.binding` wraps the C-ABI library built from `csrc/`;
`paper_2603_09221_amd.synth` draws the seeded synthetic workloads.  Nothing is imported
eagerly so that the input generators can be used without the HIP library.
"""
__all__ = ["binding", "synth"]
